// C ABI of libalch: argument validation, workspace planning and the order of kernel launches.
// Every entry point checks its arguments on the host before anything is enqueued, so all
// error paths can be exercised without a GPU.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "kernels.h"

namespace alch {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}
void clear_error() { g_error[0] = 0; }

// ---- launch tracing --------------------------------------------------------------------------
struct TraceRec {
    int kind;
    double flops, bytes;
    hipEvent_t e0, e1;
};
static std::mutex g_trace_mu;
static std::atomic<bool> g_trace_on{false};
static std::vector<TraceRec*> g_trace;
static constexpr size_t kTraceMax = 1 << 16;

TraceScope::TraceScope(int kind, double flops, double bytes, hipStream_t s) : rec(nullptr), stream(s) {
    if (!g_trace_on.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lk(g_trace_mu);
    if (g_trace.size() >= kTraceMax) return;
    TraceRec* r = new TraceRec{kind, flops, bytes, nullptr, nullptr};
    if (hipEventCreate(&r->e0) != hipSuccess || hipEventCreate(&r->e1) != hipSuccess) {
        delete r;
        return;
    }
    (void)hipEventRecord(r->e0, s);
    g_trace.push_back(r);
    rec = r;
}
TraceScope::~TraceScope() {
    if (rec) (void)hipEventRecord(static_cast<TraceRec*>(rec)->e1, stream);
}

static int check_shape(const alch_layer_shape* s) {
    if (!s) return fail(ALCH_ERR_INVALID_ARG, "shape is NULL");
    if (s->dtype != ALCH_F32 && s->dtype != ALCH_BF16) return fail(ALCH_ERR_INVALID_ARG, "bad dtype %d", (int)s->dtype);
    if (s->hidden <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 || s->ffn <= 0)
        return fail(ALCH_ERR_SHAPE, "non-positive layer dimension");
    if (s->n_q_heads % s->n_kv_heads) return fail(ALCH_ERR_SHAPE, "n_q_heads %d not a multiple of n_kv_heads %d", s->n_q_heads, s->n_kv_heads);
    if (s->head_dim % 2) return fail(ALCH_ERR_SHAPE, "head_dim %d is odd", s->head_dim);
    if (s->head_dim > 256) return fail(ALCH_ERR_UNSUPPORTED, "head_dim %d > 256", s->head_dim);
    if (s->hidden > 8192) return fail(ALCH_ERR_UNSUPPORTED, "hidden %d > 8192", s->hidden);
    if (!(s->rms_eps >= 0.f) || !(s->rope_base > 0.f)) return fail(ALCH_ERR_INVALID_ARG, "bad rms_eps / rope_base");
    return ALCH_OK;
}

static int check_batch(const alch_batch* b) {
    if (!b) return fail(ALCH_ERR_INVALID_ARG, "batch is NULL");
    if (b->n_seqs < 0 || b->total_tokens < 0 || b->max_seqlen < 0) return fail(ALCH_ERR_INVALID_ARG, "negative batch size");
    if (!b->cu_seqlens || !b->cu_seqlens_host) return fail(ALCH_ERR_INVALID_ARG, "cu_seqlens / cu_seqlens_host is NULL");
    const int32_t* cu = b->cu_seqlens_host;
    if (cu[0] != 0) return fail(ALCH_ERR_SHAPE, "cu_seqlens[0] = %d, expected 0", cu[0]);
    for (int s = 0; s < b->n_seqs; ++s) {
        const int len = cu[s + 1] - cu[s];
        if (len < 0) return fail(ALCH_ERR_SHAPE, "cu_seqlens decreases at sequence %d", s);
        if (len > b->max_seqlen) return fail(ALCH_ERR_SHAPE, "sequence %d has %d tokens > max_seqlen %d", s, len, b->max_seqlen);
    }
    if (cu[b->n_seqs] != b->total_tokens)
        return fail(ALCH_ERR_SHAPE, "cu_seqlens[n_seqs] = %d but total_tokens = %d", cu[b->n_seqs], b->total_tokens);
    if ((b->seq_prefix == nullptr) != (b->seq_prefix_host == nullptr))
        return fail(ALCH_ERR_INVALID_ARG, "seq_prefix and seq_prefix_host must be given together");
    if (b->seq_prefix_host) {
        if (b->n_seqs > kMaxPrefixSeqs) return fail(ALCH_ERR_UNSUPPORTED, "shared prefixes: more than %d sequences", kMaxPrefixSeqs);
        if (b->total_tokens > 0 && !b->positions) return fail(ALCH_ERR_INVALID_ARG, "positions must be given with seq_prefix");
        for (int s = 0; s < b->n_seqs; ++s) {
            const int p = b->seq_prefix_host[s];
            if (p < -1 || p >= s) return fail(ALCH_ERR_SHAPE, "seq_prefix[%d] = %d is not -1 or an earlier sequence", s, p);
            if (p >= 0 && b->seq_prefix_host[p] != -1) return fail(ALCH_ERR_SHAPE, "seq_prefix[%d] = %d has a prefix itself", s, p);
        }
    }
    return ALCH_OK;
}

#define REQUIRE_PTR(p, name)                                                                   \
    do {                                                                                       \
        if (!(p)) return fail(ALCH_ERR_INVALID_ARG, "%s is NULL", name);                       \
        if (!aligned16(p)) return fail(ALCH_ERR_INVALID_ARG, "%s is not 16-byte aligned", name); \
    } while (0)
#define OPTIONAL_PTR(p, name)                                                                          \
    do {                                                                                               \
        if ((p) && !aligned16(p)) return fail(ALCH_ERR_INVALID_ARG, "%s is not 16-byte aligned", name); \
    } while (0)

// ---- workspace plans -----------------------------------------------------------------------

struct LayerBwdPlan {
    void *dYm, *dGU, *Act, *Hn, *dHn, *dX2, *dO, *dQKV;
    float *delta, *partial;
    // stand-ins for record tensors the caller did not save (O, LSE, X2)
    void *O_re = nullptr, *X2_re = nullptr;
    float* LSE_re = nullptr;
    // loss-mask compaction: kept rows of dY, X2, O, G, U; compact dX2, dO; kept-row index, its inverse,
    // per-sequence counts, {n_kept, overflow}; scratch of the mask scan
    void *c_dY, *c_X2, *c_O, *c_G, *c_U, *c_dX2, *c_dO, *c_packws;
    int *c_index, *c_inv, *c_cu, *c_n;
    // adapters (rank > 0): t1 = s x A^T and t2 = s dy B, three zero-padded 64-column slots [T, 192] each;
    // the adapters' A matrices zero-padded to 64 rows and stacked per product; B transposed; partial sums of
    // the adapter gradients
    void *T1 = nullptr, *T2 = nullptr;
    void *Ap_d = nullptr, *Ap_gu = nullptr, *Ap_o = nullptr, *Ap_qkv = nullptr;  // [64,F] [128,H] [64,QD] [192,H]
    void* Bt[ALCH_N_PROJ] = {};                                                  // B_p transposed: [rank, out_p]
    float* up_scratch = nullptr;
    void* gemm_ws = nullptr;  // fp32 partial tiles of a weight-gradient product whose last round of tiles is split
    size_t bytes;
};

static LayerBwdPlan plan_layer_bwd(const alch_layer_shape& s, int T, void* ws, size_t ws_bytes, int lora_rank = 0) {
    Arena a(ws, ws_bytes);
    const size_t E = dtype_size(s.dtype);
    const size_t t = (size_t)(T > 0 ? T : 1);
    const size_t H = s.hidden, F = s.ffn, QD = (size_t)s.n_q_heads * s.head_dim, KD = (size_t)s.n_kv_heads * s.head_dim;
    LayerBwdPlan p;
    p.dYm = a.take(t * H * E);
    p.dGU = a.take(t * 2 * F * E);
    p.Act = a.take(t * F * E);
    p.Hn = a.take(t * H * E);
    p.dHn = a.take(t * H * E);
    p.dX2 = a.take(t * H * E);
    p.dO = a.take(t * QD * E);
    p.dQKV = a.take(t * (QD + 2 * KD) * E);
    p.delta = static_cast<float*>(a.take(2 * t * s.n_q_heads * sizeof(float)));  // delta, and LSE * log2(e) behind it
    p.partial = static_cast<float*>(a.take((size_t)rmsnorm_bwd_blocks(T) * H * sizeof(float)));
    p.O_re = a.take(t * QD * E);
    p.X2_re = a.take(t * H * E);
    p.LSE_re = static_cast<float*>(a.take(t * s.n_q_heads * sizeof(float)));
    p.c_dY = a.take(t * H * E); p.c_X2 = a.take(t * H * E); p.c_O = a.take(t * QD * E);
    p.c_G = a.take(t * F * E); p.c_U = a.take(t * F * E);
    p.c_dX2 = a.take(t * H * E); p.c_dO = a.take(t * QD * E);
    p.c_packws = a.take(pack_workspace_bytes(T > 0 ? T : 1));
    p.c_index = static_cast<int*>(a.take(t * sizeof(int)));
    p.c_inv = static_cast<int*>(a.take(t * sizeof(int)));
    p.c_cu = static_cast<int*>(a.take(256));
    p.c_n = static_cast<int*>(a.take(256));
    p.gemm_ws = a.take(kGemmSplitWsBytes);
    if (lora_rank > 0) {
        p.T1 = a.take(t * 3 * kLoraSlot * E);
        p.T2 = a.take(t * 3 * kLoraSlot * E);
        p.Ap_d = a.take(kLoraSlot * F * E);
        p.Ap_gu = a.take(2 * kLoraSlot * H * E);
        p.Ap_o = a.take(kLoraSlot * QD * E);
        p.Ap_qkv = a.take(3 * kLoraSlot * H * E);
        const size_t outs[ALCH_N_PROJ] = {QD, KD, KD, H, F, F, H};
        for (int i = 0; i < ALCH_N_PROJ; ++i) p.Bt[i] = a.take((size_t)lora_rank * outs[i] * E);
        // the widest group of adapter gradients formed by one launch: gate + up (dA on H twice, dB on F twice) or
        // q + k + v (dA on H three times, dB on QD + 2 KD)
        const size_t n_sum = std::max(2 * (H + F), std::max(3 * H + QD + 2 * KD, std::max(F + H, QD + H)));
        p.up_scratch = static_cast<float*>(a.take(lora_up_scratch_bytes(lora_rank, (int)n_sum)));
    }
    p.bytes = round_up(a.used, 256);
    return p;
}

struct LayerFwdPlan {
    void *Hn, *Act, *gemm_ws;
    size_t bytes;
};
static LayerFwdPlan plan_layer_fwd(const alch_layer_shape& s, int T, void* ws, size_t ws_bytes) {
    Arena a(ws, ws_bytes);
    const size_t E = dtype_size(s.dtype), t = (size_t)(T > 0 ? T : 1);
    LayerFwdPlan p;
    p.Hn = a.take(t * s.hidden * E);
    p.Act = a.take(t * s.ffn * E);
    p.gemm_ws = a.take(kGemmSplitWsBytes);
    p.bytes = round_up(a.used, 256);
    return p;
}

static constexpr int kHeadChunkRows = 8192;

struct StackPlan {
    void *Hf, *dHf, *logits, *ping, *pong, *layer_ws;
    float* row_loss;
    int* n_counted;
    float* partial;
    // loss-mask compaction of the head: counted-token mask, compacted Hf / labels / dHf, kept-row index and
    // its inverse, {n, overflow}, rows per chunk, scratch of the mask scan
    uint8_t* h_counted;
    void *h_Hf, *h_dHf, *h_packws;
    int *h_labels, *h_index, *h_inv, *h_cu, *h_n, *h_chunk_rows;
    // DPO head: log-probability and log-normaliser per item, sum and weight per slot
    float *dpo_logp, *dpo_logz, *dpo_pi, *dpo_w;
    size_t layer_ws_bytes, bytes;
};
static StackPlan plan_stack(const alch_layer_shape& s, int vocab, int T, void* ws, size_t ws_bytes, int lora_rank = 0) {
    Arena a(ws, ws_bytes);
    const size_t E = dtype_size(s.dtype), t = (size_t)(T > 0 ? T : 1), H = s.hidden;
    const size_t chunk = t < (size_t)kHeadChunkRows ? t : (size_t)kHeadChunkRows;
    StackPlan p;
    p.Hf = a.take(t * H * E);
    p.dHf = a.take(t * H * E);
    p.logits = a.take(chunk * (size_t)vocab * E);
    p.ping = a.take(t * H * E);
    p.pong = a.take(t * H * E);
    p.row_loss = static_cast<float*>(a.take(t * sizeof(float)));
    p.n_counted = static_cast<int*>(a.take(256));
    p.partial = static_cast<float*>(a.take((size_t)rmsnorm_bwd_blocks(T) * H * sizeof(float)));
    p.h_counted = static_cast<uint8_t*>(a.take(t));
    p.h_Hf = a.take(t * H * E);
    p.h_dHf = a.take(t * H * E);
    p.h_packws = a.take(pack_workspace_bytes(T > 0 ? T : 1));
    p.h_labels = static_cast<int*>(a.take(t * sizeof(int)));
    p.h_index = static_cast<int*>(a.take(t * sizeof(int)));
    p.h_inv = static_cast<int*>(a.take(t * sizeof(int)));
    p.h_cu = static_cast<int*>(a.take(256));
    p.h_n = static_cast<int*>(a.take(256));
    p.h_chunk_rows = static_cast<int*>(a.take(((t + kHeadChunkRows - 1) / kHeadChunkRows) * sizeof(int)));
    p.dpo_logp = static_cast<float*>(a.take(t * sizeof(float)));
    p.dpo_logz = static_cast<float*>(a.take(t * sizeof(float)));
    p.dpo_pi = static_cast<float*>(a.take(t * sizeof(float)));
    p.dpo_w = static_cast<float*>(a.take(t * sizeof(float)));
    p.layer_ws_bytes = plan_layer_bwd(s, T, nullptr, 0, lora_rank).bytes;
    p.layer_ws = a.take(p.layer_ws_bytes);
    p.bytes = round_up(a.used, 256);
    return p;
}

// ---- layer backward --------------------------------------------------------------------------

static GemmDesc gemm(alch_dtype dt, int M, int N, bool a_k, bool b_k) {
    GemmDesc d;
    d.M = M; d.N = N; d.a_kmajor = a_k; d.b_kmajor = b_k; d.dtype = dt;
    return d;
}
static void add_seg(GemmDesc& d, const void* A, long long lda, const void* B, long long ldb, int K) {
    d.seg[d.n_seg++] = GemmSeg{A, B, K, lda, ldb};
}
static void add_out(GemmDesc& d, void* C, int m_begin, long long ldc) { d.out[d.n_out++] = GemmOut{C, m_begin, ldc}; }

static inline const char* at(const void* p, size_t elems, size_t E) { return static_cast<const char*>(p) + elems * E; }
static inline char* at(void* p, size_t elems, size_t E) { return static_cast<char*>(p) + elems * E; }

// Activation pointers may be NULL only when the batch holds no token.
#define REQUIRE_ACT(p, name, T)                   \
    do {                                          \
        if ((T) > 0) REQUIRE_PTR(p, name);        \
        else OPTIONAL_PTR(p, name);               \
    } while (0)

static int check_saved_weights(const alch_saved* sv, const alch_weights* w, int T) {
    if (!sv || !w) return fail(ALCH_ERR_INVALID_ARG, "saved / weights is NULL");
    REQUIRE_ACT(sv->X, "saved.X", T); REQUIRE_ACT(sv->Q, "saved.Q", T);
    REQUIRE_ACT(sv->K, "saved.K", T); REQUIRE_ACT(sv->V, "saved.V", T);
    // X2, O, LSE, G and U may be NULL: they are then recomputed from the rest of the record
    OPTIONAL_PTR(sv->G, "saved.G"); OPTIONAL_PTR(sv->U, "saved.U");
    OPTIONAL_PTR(sv->X2, "saved.X2"); OPTIONAL_PTR(sv->O, "saved.O"); OPTIONAL_PTR(sv->LSE, "saved.LSE");
    REQUIRE_PTR(w->Wq, "weights.Wq"); REQUIRE_PTR(w->Wk, "weights.Wk"); REQUIRE_PTR(w->Wv, "weights.Wv");
    REQUIRE_PTR(w->Wo, "weights.Wo"); REQUIRE_PTR(w->Wg, "weights.Wg"); REQUIRE_PTR(w->Wu, "weights.Wu");
    REQUIRE_PTR(w->Wd, "weights.Wd"); REQUIRE_PTR(w->g1, "weights.g1"); REQUIRE_PTR(w->g2, "weights.g2");
    if (sv->weights_version != w->weights_version)
        return fail(ALCH_ERR_STALE, "record was captured under weights version %llu, weights are version %llu",
                    (unsigned long long)sv->weights_version, (unsigned long long)w->weights_version);
    return ALCH_OK;
}

static int check_wgrads(const alch_wgrads* g) {
    if (!g) return ALCH_OK;
    OPTIONAL_PTR(g->dWq, "wgrads.dWq"); OPTIONAL_PTR(g->dWk, "wgrads.dWk"); OPTIONAL_PTR(g->dWv, "wgrads.dWv");
    OPTIONAL_PTR(g->dWo, "wgrads.dWo"); OPTIONAL_PTR(g->dWg, "wgrads.dWg"); OPTIONAL_PTR(g->dWu, "wgrads.dWu");
    OPTIONAL_PTR(g->dWd, "wgrads.dWd"); OPTIONAL_PTR(g->dg1, "wgrads.dg1"); OPTIONAL_PTR(g->dg2, "wgrads.dg2");
    return ALCH_OK;
}

// Enqueues steps of one layer's backward pass; arguments already validated.
static int layer_backward_enqueue(const alch_layer_shape& s, const alch_batch& b, const alch_saved& sv_in,
                                  const alch_weights& w, const void* dY, const uint8_t* loss_mask, void* dX,
                                  const alch_wgrads* wg, const LayerBwdPlan& p, hipStream_t st,
                                  const alch_lora* lo = nullptr, const alch_lora_grads* lg = nullptr) {
    const alch_dtype dt = s.dtype;
    const size_t E = dtype_size(dt);
    const int T = b.total_tokens, H = s.hidden, F = s.ffn, D = s.head_dim;
    const int QD = s.n_q_heads * D, KD = s.n_kv_heads * D, QKV = QD + 2 * KD;
    // every product may split a half-empty last round of tiles (short batches: all tiles) into the plan's scratch
    auto gemm_ws = [&](alch_dtype t, int M, int N, bool a_k, bool b_k) {
        GemmDesc d = gemm(t, M, N, a_k, b_k);
        d.split_ws = p.gemm_ws;
        d.split_ws_bytes = kGemmSplitWsBytes;
        return d;
    };

    // A record without O / LSE / X2 (Section 4.3.2: recompute instead of load): attention forward on the saved
    // post-RoPE Q, K, V gives O and LSE; X2 = X + O Wo^T (sum in fp32, one rounding, as the forward does).
    alch_saved sv = sv_in;
    if (T > 0 && (!sv.O || !sv.LSE)) {
        ALCH_TRY(launch_attn_fwd(dt, sv.Q, sv.K, sv.V, p.O_re, p.LSE_re, T, b.n_seqs, b.max_seqlen, b.cu_seqlens,
                                 b.cu_seqlens_host, b.seq_prefix, b.seq_prefix_host, 0, s.n_q_heads, s.n_kv_heads, D, st));
        sv.O = p.O_re;
        sv.LSE = p.LSE_re;
    }
    if (T > 0 && !sv.X2) {
        if (lo && lo->A[ALCH_PROJ_O])
            return fail(ALCH_ERR_UNSUPPORTED, "saved.X2 must be given when the output projection carries an adapter");
        ALCH_TRY(launch_masked_copy(dt, sv.X, nullptr, p.X2_re, T, H, st));
        GemmDesc d;
        d.M = T; d.N = H; d.a_kmajor = true; d.b_kmajor = true; d.dtype = dt;
        d.seg[d.n_seg++] = GemmSeg{sv.O, w.Wo, QD, QD, QD};
        d.out[d.n_out++] = GemmOut{p.X2_re, 0, H};
        d.accumulate = 1;
        ALCH_TRY(launch_gemm(d, st));
        sv.X2 = p.X2_re;
    }
    // A record without G / U: the MLP pre-activations are H2 Wg^T, H2 Wu^T with H2 the normalised X2, computed
    // below on the rows the MLP backward will read (all T, or the kept rows under a loss mask).
    const bool re_gu = T > 0 && (!sv.G || !sv.U);
    if (re_gu && lo && (lo->A[ALCH_PROJ_G] || lo->A[ALCH_PROJ_U]))
        return fail(ALCH_ERR_UNSUPPORTED, "saved.G and saved.U must be given when the gate or up projection carries an adapter");
    bool hn_ready = false;  // p.Hn already holds the normalised X2 rows
    auto recompute_gu = [&](const void* x2, const int* rows_dev) -> int {
        ALCH_TRY(launch_rmsnorm_fwd(dt, x2, w.g2, p.Hn, T, H, s.rms_eps, st, rows_dev));
        hn_ready = true;
        const void* Wm[2] = {w.Wg, w.Wu};
        void* om[2] = {p.c_G, p.c_U};
        const void* have[2] = {sv.G, sv.U};
        for (int i = 0; i < 2; ++i) {
            if (have[i]) continue;
            GemmDesc d;
            d.M = T; d.N = F; d.a_kmajor = true; d.b_kmajor = true; d.dtype = dt;
            d.m_dev = rows_dev;
            d.seg[d.n_seg++] = GemmSeg{p.Hn, Wm[i], H, H, H};
            d.out[d.n_out++] = GemmOut{om[i], 0, F};
            ALCH_TRY(launch_gemm(d, st));
        }
        return ALCH_OK;
    };
    const int acc = wg ? (wg->accumulate != 0) : 0;
    static const alch_wgrads none = {};
    const alch_wgrads& g = wg ? *wg : none;

    // ---- adapters.  For an adapted projection y = x W^T + s (x A^T) B^T with incoming gradient dy:
    //   t2 = s dy B  [T, r]      -> data gradient  dx += t2 A   (an extra operand pair of the projection's
    //                               data-gradient product: t2 zero-padded to 64 columns, A to 64 rows)
    //                            -> dA = t2^T x
    //   t1 = s x A^T [T, r]      -> dB = dy^T t1
    const int r = lo ? lo->rank : 0;
    const int lacc = lg ? (lg->accumulate != 0) : 0;
    const long long ldt2 = 3 * kLoraSlot;
    auto has = [&](int pj) { return lo && lo->A[pj] && lo->B[pj]; };
    auto wants = [&](int pj) { return has(pj) && lg && (lg->dA[pj] || lg->dB[pj]); };
    // t2 of up to three projections (first one pj0) into slots 0, 1, ... (zeros where there is no adapter)
    auto down_t2 = [&](int pj0, int n, const void* const* dy, long long lddy, const int* out_p) {
        LoraDown jobs[3];
        for (int i = 0; i < n; ++i) {
            const bool on = has(pj0 + i);
            jobs[i] = LoraDown{dy[i], lddy, out_p[i], on ? p.Bt[pj0 + i] : nullptr, out_p[i], on ? r : 0,
                               const_cast<char*>(at(p.T2, (size_t)i * kLoraSlot, E))};
        }
        return launch_lora_down(dt, jobs, n, T, lo->scale, ldt2, kLoraSlot, st);
    };
    if (lo) {  // operand preparation for the whole layer, one launch
        LoraPrepParams pp;
        int nj = 0;
        auto pad = [&](int pj, void* base, int slot, int in_p) {
            pp.job[nj++] = LoraPrepJob{has(pj) ? lo->A[pj] : nullptr, const_cast<char*>(at(base, (size_t)slot * kLoraSlot * in_p, E)),
                                       r, in_p, kLoraSlot, 0};
        };
        pad(ALCH_PROJ_D, p.Ap_d, 0, F);
        pad(ALCH_PROJ_G, p.Ap_gu, 0, H);
        pad(ALCH_PROJ_U, p.Ap_gu, 1, H);
        pad(ALCH_PROJ_O, p.Ap_o, 0, QD);
        for (int i = 0; i < 3; ++i) pad(ALCH_PROJ_Q + i, p.Ap_qkv, i, H);
        const int outs[ALCH_N_PROJ] = {QD, KD, KD, H, F, F, H};
        for (int pj = 0; pj < ALCH_N_PROJ; ++pj)
            if (has(pj)) pp.job[nj++] = LoraPrepJob{lo->B[pj], p.Bt[pj], r, outs[pj], r, 1};
        ALCH_TRY(launch_lora_prep(dt, pp, nj, st));
    }
    // Adapter gradients of the n <= 3 projections pj0, pj0+1, .. that share the input x [T, in_p]; dy[i] [T, out_p[i]]
    // with row stride lddy; t2 of projection pj0+i sits in slot i.  One launch forms the t1 of all of them, one pair
    // of launches all their dA and dB.
    auto adapter_grads = [&](int pj0, int n, const void* x, long long ldx, int in_p, const void* const* dy, long long lddy,
                             const int* out_p) -> int {
        LoraDown dj[3];
        LoraUp uj[kLoraUpJobs];
        int nd = 0, nu = 0;
        const long long ldt1 = 3 * kLoraSlot;
        for (int i = 0; i < n; ++i) {
            const int pj = pj0 + i;
            if (!wants(pj)) continue;
            if (lg->dB[pj]) {
                char* t1 = at(p.T1, (size_t)nd * kLoraSlot, E);
                dj[nd++] = LoraDown{x, ldx, in_p, lo->A[pj], in_p, r, t1};
                uj[nu++] = LoraUp{t1, ldt1, dy[i], lddy, out_p[i], lg->dB[pj], r, 1};
            }
            if (lg->dA[pj]) uj[nu++] = LoraUp{at(p.T2, (size_t)i * kLoraSlot, E), ldt2, x, ldx, in_p, lg->dA[pj], in_p, 0};
        }
        if (nd) ALCH_TRY(launch_lora_down(dt, dj, nd, T, lo->scale, ldt1, kLoraSlot, st));
        if (nu) ALCH_TRY(launch_lora_up(dt, uj, nu, T, r, 1.f, lacc, p.up_scratch, st));
        return ALCH_OK;
    };

    // Loss mask.  Rows of dY whose mask byte is 0 count as zero.  Everything from the MLP down to the
    // attention output projection is row-local, so those rows contribute nothing there and receive nothing:
    //   compact mode (bf16, matrix-core shapes, no adapters): the kept rows of dY, X2, O, G, U are gathered
    //     into dense [n, width] tensors, the row-local part runs on n rows (n stays on the device: the
    //     products take their row or contraction count from device memory), and dX2, dO are scattered back
    //     into zero-filled [T, width] tensors for the attention backward, which is dense in the keys;
    //   otherwise dY is copied once with the masked rows zeroed and every step runs on all T rows.
    // (the compacted products take their sizes from device memory, which only the matrix-core kernel supports:
    // its 2 GiB operand limit, reached first by [dG | dU], is part of the decision, taken before anything is enqueued)
    const bool compact = loss_mask && T > 0 && !lo && dt == ALCH_BF16 && H % 64 == 0 && F % 64 == 0 && QD % 64 == 0 &&
                         aligned16(dY) && (long long)T * 2 * F * (long long)E < (1LL << 31);
    const void *mY = dY, *mX2 = sv.X2, *mO = sv.O, *mG = sv.G, *mU = sv.U;  // inputs of the row-local part
    void *mdX2 = p.dX2, *mdO = p.dO;                                      // its outputs
    const int* ndev = nullptr;                                              // device-resident row count
    if (compact) {
        alch_stream rows[5] = {{dY, p.c_dY, (size_t)H * E, (size_t)H * E}, {sv.X2, p.c_X2, (size_t)H * E, (size_t)H * E},
                               {sv.O, p.c_O, (size_t)QD * E, (size_t)QD * E}};
        int n_rows = 3;
        if (sv.G) rows[n_rows++] = alch_stream{sv.G, p.c_G, (size_t)F * E, (size_t)F * E};
        if (sv.U) rows[n_rows++] = alch_stream{sv.U, p.c_U, (size_t)F * E, (size_t)F * E};
        // (per-sequence counts are not needed: zero sequences asked for, one boundary written)
        ALCH_TRY(launch_pack(loss_mask, T, b.cu_seqlens, 0, n_rows, rows, T, p.c_index, p.c_cu, p.c_n, p.c_packws, st, false));
        ALCH_TRY(launch_rank_of_kept(p.c_index, p.c_n, p.c_inv, T, st));
        mY = p.c_dY; mX2 = p.c_X2; mO = p.c_O; mG = p.c_G; mU = p.c_U;
        mdX2 = p.c_dX2; mdO = p.c_dO;
        ndev = p.c_n;
        if (re_gu) ALCH_TRY(recompute_gu(mX2, ndev));
    } else {
        if (loss_mask) {
            ALCH_TRY(launch_masked_copy(dt, dY, loss_mask, p.dYm, T, H, st));
            mY = p.dYm;
        }
        if (re_gu) {
            ALCH_TRY(recompute_gu(sv.X2, nullptr));
            if (!sv.G) mG = p.c_G;
            if (!sv.U) mU = p.c_U;
        }
    }

    // MLP down projection: dAct = dY Wd, fused with the SwiGLU gradient -> [dG | dU] and Act
    if (has(ALCH_PROJ_D)) {
        const void* dys[1] = {mY};
        const int outs1[1] = {H};
        ALCH_TRY(down_t2(ALCH_PROJ_D, 1, dys, H, outs1));
    }
    {
        GemmDesc d = gemm_ws(dt, T, F, true, false);
        d.m_dev = ndev;
        add_seg(d, mY, H, w.Wd, F, H);
        if (has(ALCH_PROJ_D)) add_seg(d, p.T2, ldt2, p.Ap_d, F, kLoraSlot);
        add_out(d, p.dGU, 0, 2 * (long long)F);
        d.epilogue = kEpiSwigluBwd;
        d.G = mG; d.U = mU; d.ldgu = F;
        d.act_out = (g.dWd || wants(ALCH_PROJ_D)) ? p.Act : nullptr;
        ALCH_TRY(launch_gemm(d, st));
    }
    if (g.dWd) {  // dWd = dY^T Act
        GemmDesc d = gemm_ws(dt, H, F, false, false);
        d.k_dev = ndev;
        add_seg(d, mY, H, p.Act, F, T);
        add_out(d, g.dWd, 0, F);
        d.accumulate = acc;
        ALCH_TRY(launch_gemm(d, st));
    }
    {
        const void* dys[1] = {mY};
        const int outs1[1] = {H};
        ALCH_TRY(adapter_grads(ALCH_PROJ_D, 1, p.Act, F, F, dys, H, outs1));
    }
    const bool lora_gu = has(ALCH_PROJ_G) || has(ALCH_PROJ_U);
    if (lora_gu) {
        const void* dys[2] = {p.dGU, at(p.dGU, F, E)};
        const int outs2[2] = {F, F};
        ALCH_TRY(down_t2(ALCH_PROJ_G, 2, dys, 2 * (long long)F, outs2));
    }
    {  // dH2 = dG Wg + dU Wu
        GemmDesc d = gemm_ws(dt, T, H, true, false);
        d.m_dev = ndev;
        add_seg(d, p.dGU, 2 * (long long)F, w.Wg, H, F);
        add_seg(d, at(p.dGU, F, E), 2 * (long long)F, w.Wu, H, F);
        if (lora_gu) add_seg(d, p.T2, ldt2, p.Ap_gu, H, 2 * kLoraSlot);
        add_out(d, p.dHn, 0, H);
        ALCH_TRY(launch_gemm(d, st));
    }
    // dX2 = dY + RMSNorm-2 backward(dH2); dg2.  The same pass over X2 leaves H2 for the weight and adapter gradients
    // of the gate and up projections (unless the record completion above already formed it).
    {
        const bool need_h2 = !hn_ready && (g.dWg || g.dWu || wants(ALCH_PROJ_G) || wants(ALCH_PROJ_U));
        ALCH_TRY(launch_rmsnorm_bwd(dt, p.dHn, mX2, w.g2, mY, nullptr, mdX2, g.dg2, acc, p.partial, T, H, s.rms_eps, st, ndev,
                                    need_h2 ? p.Hn : nullptr));
    }
    {
        const void* dys[2] = {p.dGU, at(p.dGU, F, E)};
        const int outs2[2] = {F, F};
        ALCH_TRY(adapter_grads(ALCH_PROJ_G, 2, p.Hn, H, H, dys, 2 * (long long)F, outs2));
    }
    if (g.dWg || g.dWu) {  // [dWg; dWu] = [dG | dU]^T H2
        if (g.dWg && g.dWu) {
            GemmDesc d = gemm_ws(dt, 2 * F, H, false, false);
            d.k_dev = ndev;
            add_seg(d, p.dGU, 2 * (long long)F, p.Hn, H, T);
            add_out(d, g.dWg, 0, H);
            add_out(d, g.dWu, F, H);
            d.accumulate = acc;
            if (F % 256 == 0) {
                ALCH_TRY(launch_gemm(d, st));
            } else {
                d.M = F; d.n_out = 1;
                ALCH_TRY(launch_gemm(d, st));
                d.seg[0].A = at(p.dGU, F, E); d.out[0].C = g.dWu;
                ALCH_TRY(launch_gemm(d, st));
            }
        } else {
            GemmDesc d = gemm_ws(dt, F, H, false, false);
            d.k_dev = ndev;
            add_seg(d, g.dWg ? p.dGU : at(p.dGU, F, E), 2 * (long long)F, p.Hn, H, T);
            add_out(d, g.dWg ? g.dWg : g.dWu, 0, H);
            d.accumulate = acc;
            ALCH_TRY(launch_gemm(d, st));
        }
    }

    if (has(ALCH_PROJ_O)) {
        const void* dys[1] = {mdX2};
        const int outs1[1] = {H};
        ALCH_TRY(down_t2(ALCH_PROJ_O, 1, dys, H, outs1));
    }
    {  // dO = dX2 Wo
        GemmDesc d = gemm_ws(dt, T, QD, true, false);
        d.m_dev = ndev;
        add_seg(d, mdX2, H, w.Wo, QD, H);
        if (has(ALCH_PROJ_O)) add_seg(d, p.T2, ldt2, p.Ap_o, QD, kLoraSlot);
        add_out(d, mdO, 0, QD);
        ALCH_TRY(launch_gemm(d, st));
    }
    {
        const void* dys[1] = {mdX2};
        const int outs1[1] = {H};
        ALCH_TRY(adapter_grads(ALCH_PROJ_O, 1, mO, QD, QD, dys, H, outs1));
    }
    if (g.dWo) {  // dWo = dX2^T O
        GemmDesc d = gemm_ws(dt, H, QD, false, false);
        d.k_dev = ndev;
        add_seg(d, mdX2, H, mO, QD, T);
        add_out(d, g.dWo, 0, QD);
        d.accumulate = acc;
        ALCH_TRY(launch_gemm(d, st));
    }

    if (compact) {  // back to [T, width]: zeros in the masked rows
        ALCH_TRY(launch_scatter_rows(p.c_dO, p.c_inv, p.dO, T, (size_t)QD * E, st));
        ALCH_TRY(launch_scatter_rows(p.c_dX2, p.c_inv, p.dX2, T, (size_t)H * E, st));
    }

    // attention backward from saved Q, K, V, O, LSE -> [dQ | dK | dV] with RoPE backward applied to dQ, dK
    {
        AttnArgs a;
        a.dtype = dt; a.T = T; a.n_seqs = b.n_seqs; a.max_seqlen = b.max_seqlen;
        a.Hq = s.n_q_heads; a.Hkv = s.n_kv_heads; a.D = D;
        a.cu_seqlens = b.cu_seqlens; a.cu_seqlens_host = b.cu_seqlens_host;
        a.prefix = b.seq_prefix; a.prefix_host = b.seq_prefix_host;
        a.Q = sv.Q; a.K = sv.K; a.V = sv.V; a.O = sv.O; a.dO = p.dO; a.LSE = sv.LSE; a.delta = p.delta;
        a.dQ = p.dQKV; a.dK = at(p.dQKV, QD, E); a.dV = at(p.dQKV, QD + KD, E); a.ld_dqkv = QKV;
        a.positions = b.positions; a.rope_base = s.rope_base;
        ALCH_TRY(launch_attn_bwd(a, st));
    }

    const bool lora_qkv = has(ALCH_PROJ_Q) || has(ALCH_PROJ_K) || has(ALCH_PROJ_V);
    if (lora_qkv) {
        const void* dys[3] = {p.dQKV, at(p.dQKV, QD, E), at(p.dQKV, QD + KD, E)};
        const int outs3[3] = {QD, KD, KD};
        ALCH_TRY(down_t2(ALCH_PROJ_Q, 3, dys, QKV, outs3));
    }
    {  // dH1 = dQ Wq + dK Wk + dV Wv
        GemmDesc d = gemm_ws(dt, T, H, true, false);
        add_seg(d, p.dQKV, QKV, w.Wq, H, QD);
        add_seg(d, at(p.dQKV, QD, E), QKV, w.Wk, H, KD);
        add_seg(d, at(p.dQKV, QD + KD, E), QKV, w.Wv, H, KD);
        if (lora_qkv) add_seg(d, p.T2, ldt2, p.Ap_qkv, H, 3 * kLoraSlot);
        add_out(d, p.dHn, 0, H);
        ALCH_TRY(launch_gemm(d, st));
    }
    // dX = dX2 + RMSNorm-1 backward(dH1); dg1.  The same pass over X leaves H1 for the weight and adapter gradients of
    // the q, k, v projections.
    {
        const bool need_h1 = g.dWq || g.dWk || g.dWv || wants(ALCH_PROJ_Q) || wants(ALCH_PROJ_K) || wants(ALCH_PROJ_V);
        ALCH_TRY(launch_rmsnorm_bwd(dt, p.dHn, sv.X, w.g1, p.dX2, nullptr, dX, g.dg1, acc, p.partial, T, H, s.rms_eps, st, nullptr,
                                    need_h1 ? p.Hn : nullptr));
    }
    {
        const void* dys[3] = {p.dQKV, at(p.dQKV, QD, E), at(p.dQKV, QD + KD, E)};
        const int outs3[3] = {QD, KD, KD};
        ALCH_TRY(adapter_grads(ALCH_PROJ_Q, 3, p.Hn, H, H, dys, QKV, outs3));
    }
    if (g.dWq || g.dWk || g.dWv) {  // dW{q,k,v} = d{Q,K,V}^T H1
        if (g.dWq && g.dWk && g.dWv && QD % 256 == 0 && KD % 256 == 0) {
            GemmDesc d = gemm_ws(dt, QKV, H, false, false);
            add_seg(d, p.dQKV, QKV, p.Hn, H, T);
            add_out(d, g.dWq, 0, H);
            add_out(d, g.dWk, QD, H);
            add_out(d, g.dWv, QD + KD, H);
            d.accumulate = acc;
            ALCH_TRY(launch_gemm(d, st));
        } else {
            void* outs[3] = {g.dWq, g.dWk, g.dWv};
            const int off[3] = {0, QD, QD + KD}, rows[3] = {QD, KD, KD};
            for (int i = 0; i < 3; ++i) {
                if (!outs[i]) continue;
                GemmDesc d = gemm_ws(dt, rows[i], H, false, false);
                add_seg(d, at(p.dQKV, off[i], E), QKV, p.Hn, H, T);
                add_out(d, outs[i], 0, H);
                d.accumulate = acc;
                ALCH_TRY(launch_gemm(d, st));
            }
        }
    }
    return ALCH_OK;
}

// (query, key) pairs per query head: causal inside a sequence, all keys of its prefix
double attn_pairs(int n_seqs, const int* cu_host, const int* prefix_host) {
    double pairs = 0;
    for (int s = 0; s < n_seqs; ++s) {
        const double n = cu_host[s + 1] - cu_host[s];
        pairs += n * (n + 1) / 2;
        if (prefix_host && prefix_host[s] >= 0) pairs += n * (cu_host[prefix_host[s] + 1] - cu_host[prefix_host[s]]);
    }
    return pairs;
}

int launch_attn_bwd(const AttnArgs& a, hipStream_t stream) {
    TraceScope ts(kTraceAttnBwd, 10.0 * a.D * a.Hq * attn_pairs(a.n_seqs, a.cu_seqlens_host, a.prefix_host), 0.0, stream);
    if (attn_mfma_supported(a)) return launch_attn_bwd_mfma(a, stream);  // delta and RoPE backward fused
    ALCH_TRY(launch_attn_delta(a.dtype, a.dO, a.O, a.delta, a.T, a.Hq, a.D, stream));
    ALCH_TRY(launch_attn_bwd_generic(a, stream));
    if (a.rope_base > 0.f)
        ALCH_TRY(launch_rope(a.dtype, a.dQ, a.ld_dqkv, a.T, a.Hq + a.Hkv, a.D, a.positions, a.cu_seqlens, a.n_seqs,
                             a.rope_base, -1.f, stream));
    return ALCH_OK;
}

}  // namespace alch

using namespace alch;

extern "C" {

int alch_trace_enable(int32_t enable) {
    std::lock_guard<std::mutex> lk(g_trace_mu);
    g_trace_on.store(enable != 0, std::memory_order_release);
    return ALCH_OK;
}

int alch_trace_collect(alch_trace_record* out, int32_t max_records, int32_t* n_out) {
    clear_error();
    if (!n_out || (max_records > 0 && !out) || max_records < 0) return fail(ALCH_ERR_INVALID_ARG, "bad trace buffer");
    std::lock_guard<std::mutex> lk(g_trace_mu);
    int n = 0;
    int rc = ALCH_OK;
    for (TraceRec* r : g_trace) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r->e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r->e0, r->e1);
        if (e != hipSuccess) rc = fail(ALCH_ERR_HIP, "trace event: %s", hipGetErrorString(e));
        if (n < max_records && e == hipSuccess) out[n++] = alch_trace_record{r->kind, r->flops, r->bytes, ms};
        (void)hipEventDestroy(r->e0);
        (void)hipEventDestroy(r->e1);
        delete r;
    }
    g_trace.clear();
    *n_out = n;
    return rc;
}

const char* alch_last_error(void) { return g_error; }
const char* alch_version(void) { return "alch 0.1 (gfx950)"; }

size_t alch_gemm_workspace_bytes(void) { return kGemmSplitWsBytes; }

int alch_gemm(alch_dtype dtype, int32_t M, int32_t N, int32_t a_kmajor, int32_t b_kmajor, int32_t n_terms,
              const alch_gemm_term* terms, void* C, int64_t ldc, int32_t accumulate, void* hip_stream) {
    return alch_gemm_ws(dtype, M, N, a_kmajor, b_kmajor, n_terms, terms, C, ldc, accumulate, nullptr, 0, hip_stream);
}

int alch_gemm_ws(alch_dtype dtype, int32_t M, int32_t N, int32_t a_kmajor, int32_t b_kmajor, int32_t n_terms,
                 const alch_gemm_term* terms, void* C, int64_t ldc, int32_t accumulate, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
    clear_error();
    if (workspace && !aligned16(workspace)) return fail(ALCH_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    if (dtype != ALCH_F32 && dtype != ALCH_BF16) return fail(ALCH_ERR_INVALID_ARG, "bad dtype %d", (int)dtype);
    if (M < 0 || N < 0) return fail(ALCH_ERR_SHAPE, "negative M or N");
    if (n_terms < 1 || n_terms > kMaxGemmSegs || !terms) return fail(ALCH_ERR_INVALID_ARG, "n_terms must be 1..%d and terms non-NULL", kMaxGemmSegs);
    if (!C || ldc < N) return fail(ALCH_ERR_INVALID_ARG, "C is NULL or ldc < N");
    GemmDesc d = gemm(dtype, M, N, a_kmajor != 0, b_kmajor != 0);
    for (int i = 0; i < n_terms; ++i) {
        const alch_gemm_term& t = terms[i];
        if (t.K < 0) return fail(ALCH_ERR_SHAPE, "term %d: K < 0", i);
        if (t.K > 0 && (!t.A || !t.B)) return fail(ALCH_ERR_INVALID_ARG, "term %d: NULL operand", i);
        if (t.lda < (a_kmajor ? t.K : M) || t.ldb < (b_kmajor ? t.K : N))
            return fail(ALCH_ERR_SHAPE, "term %d: leading dimension smaller than the row length", i);
        add_seg(d, t.A, t.lda, t.B, t.ldb, t.K);
    }
    add_out(d, C, 0, ldc);
    d.accumulate = accumulate != 0;
    d.split_ws = workspace;
    d.split_ws_bytes = workspace ? workspace_bytes : 0;
    return launch_gemm(d, static_cast<hipStream_t>(hip_stream));
}

size_t alch_capture_pack_workspace_bytes(int32_t total_tokens) { return pack_workspace_bytes(total_tokens); }

static int check_streams(int32_t n_streams, const alch_stream* streams, int T, int64_t dst_capacity_rows);

int alch_capture_pack(const alch_batch* batch, const uint8_t* keep_mask, int32_t n_streams,
                      const alch_stream* streams, int64_t dst_capacity_rows, int32_t* kept_index, int32_t* cu_kept,
                      int32_t* n_kept_and_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    clear_error();
    ALCH_TRY(check_batch(batch));
    if (batch->total_tokens > 0 && !keep_mask) return fail(ALCH_ERR_INVALID_ARG, "keep_mask is NULL");
    OPTIONAL_PTR(keep_mask, "keep_mask");
    ALCH_TRY(check_streams(n_streams, streams, batch->total_tokens, dst_capacity_rows));
    if (dst_capacity_rows > 0 && !kept_index) return fail(ALCH_ERR_INVALID_ARG, "kept_index is NULL");
    if (!cu_kept || !n_kept_and_status) return fail(ALCH_ERR_INVALID_ARG, "cu_kept / n_kept_and_status is NULL");
    const size_t need = pack_workspace_bytes(batch->total_tokens);
    if (!workspace || workspace_bytes < need) return fail(ALCH_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", workspace_bytes, need);
    return launch_pack(keep_mask, batch->total_tokens, batch->cu_seqlens, batch->n_seqs, n_streams, streams,
                       dst_capacity_rows, kept_index, cu_kept, n_kept_and_status, workspace,
                       static_cast<hipStream_t>(hip_stream));
}

// ---- capture/pack without a workspace argument ------------------------------------------------
// The scan's block counters live in a file-scope device array instead of caller memory.  The array's
// name is only a host-side handle: its device address is looked up once per device and that address is
// what the kernels receive.
static constexpr size_t kPackScratchBytes = 64 * 1024;
static constexpr int kPackScratchMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kPackScratchBytes];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kPackScratchMaxDevices] = {};

static int pack_scratch_for_current_device(void** out) {
    int dev = -1;
    ALCH_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kPackScratchMaxDevices) return fail(ALCH_ERR_UNSUPPORTED, "device ordinal %d >= %d", dev, kPackScratchMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        ALCH_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ALCH_ERR_HIP, "hipGetSymbolAddress returned a NULL address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ALCH_OK;
}

size_t alch_capture_pack_static_max_tokens(void) {
    // largest T whose scan scratch (pack_workspace_bytes) fits the array
    long long lo = 0, hi = INT32_MAX;
    while (lo < hi) {
        long long mid = (lo + hi + 1) / 2;
        if (pack_workspace_bytes((int)mid) <= kPackScratchBytes) lo = mid; else hi = mid - 1;
    }
    return (size_t)lo;
}

int alch_capture_pack_static(const alch_batch* batch, const uint8_t* keep_mask, int32_t n_streams,
                             const alch_stream* streams, int64_t dst_capacity_rows, int32_t* kept_index,
                             int32_t* cu_kept, int32_t* n_kept_and_status, void* hip_stream) {
    clear_error();
    ALCH_TRY(check_batch(batch));
    if (batch->total_tokens > 0 && !keep_mask) return fail(ALCH_ERR_INVALID_ARG, "keep_mask is NULL");
    OPTIONAL_PTR(keep_mask, "keep_mask");
    ALCH_TRY(check_streams(n_streams, streams, batch->total_tokens, dst_capacity_rows));
    if (dst_capacity_rows > 0 && !kept_index) return fail(ALCH_ERR_INVALID_ARG, "kept_index is NULL");
    if (!cu_kept || !n_kept_and_status) return fail(ALCH_ERR_INVALID_ARG, "cu_kept / n_kept_and_status is NULL");
    const size_t need = pack_workspace_bytes(batch->total_tokens);
    if (need > kPackScratchBytes)
        return fail(ALCH_ERR_UNSUPPORTED, "total_tokens %d exceeds the %zu tokens the built-in scratch (%zu bytes) serves; "
                    "use alch_capture_pack with a workspace", batch->total_tokens, alch_capture_pack_static_max_tokens(),
                    kPackScratchBytes);
    void* ws = nullptr;
    ALCH_TRY(pack_scratch_for_current_device(&ws));
    // Nothing in the scratch has to start at zero: the count kernel writes every block counter the later
    // kernels read, so the contents an earlier call left behind are never seen.
    return launch_pack(keep_mask, batch->total_tokens, batch->cu_seqlens, batch->n_seqs, n_streams, streams,
                       dst_capacity_rows, kept_index, cu_kept, n_kept_and_status, ws,
                       static_cast<hipStream_t>(hip_stream));
}

static int check_streams(int32_t n_streams, const alch_stream* streams, int T, int64_t dst_capacity_rows) {
    if (n_streams < 0) return fail(ALCH_ERR_INVALID_ARG, "n_streams < 0");
    if (n_streams > 0 && !streams) return fail(ALCH_ERR_INVALID_ARG, "streams is NULL");
    if (dst_capacity_rows < 0) return fail(ALCH_ERR_INVALID_ARG, "dst_capacity_rows < 0");
    for (int k = 0; k < n_streams; ++k) {
        const alch_stream& s = streams[k];
        if (s.row_bytes == 0 || s.row_bytes % 4) return fail(ALCH_ERR_SHAPE, "stream %d: row_bytes %zu not a positive multiple of 4", k, s.row_bytes);
        if (s.src_row_stride_bytes < s.row_bytes || s.src_row_stride_bytes % 4)
            return fail(ALCH_ERR_SHAPE, "stream %d: src_row_stride_bytes %zu < row_bytes or not a multiple of 4", k, s.src_row_stride_bytes);
        if ((T > 0 && !s.src) || (dst_capacity_rows > 0 && !s.dst)) return fail(ALCH_ERR_INVALID_ARG, "stream %d: NULL src or dst", k);
        if ((reinterpret_cast<uintptr_t>(s.src) | reinterpret_cast<uintptr_t>(s.dst)) & 3u)
            return fail(ALCH_ERR_INVALID_ARG, "stream %d: src or dst not 4-byte aligned", k);
    }
    return ALCH_OK;
}

int alch_capture_gather(const alch_batch* batch, int32_t n_streams, const alch_stream* streams, int64_t dst_capacity_rows,
                        const int32_t* kept_index, const int32_t* n_kept_and_status, void* hip_stream) {
    clear_error();
    ALCH_TRY(check_batch(batch));
    ALCH_TRY(check_streams(n_streams, streams, batch->total_tokens, dst_capacity_rows));
    if (dst_capacity_rows > 0 && !kept_index) return fail(ALCH_ERR_INVALID_ARG, "kept_index is NULL");
    if (!n_kept_and_status) return fail(ALCH_ERR_INVALID_ARG, "n_kept_and_status is NULL");
    return launch_pack_gather(batch->total_tokens, n_streams, streams, dst_capacity_rows, kept_index, n_kept_and_status,
                              static_cast<hipStream_t>(hip_stream));
}

size_t alch_layer_backward_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens, int32_t max_seqlen) {
    (void)max_seqlen;
    if (!shape || check_shape(shape) != ALCH_OK || total_tokens < 0) return 0;
    return plan_layer_bwd(*shape, total_tokens, nullptr, 0).bytes;
}

int alch_layer_backward(const alch_layer_shape* shape, const alch_batch* batch, const alch_saved* saved,
                        const alch_weights* weights, const void* dY, const uint8_t* loss_mask, void* dX,
                        const alch_wgrads* wgrads, void* workspace, size_t workspace_bytes, void* hip_stream) {
    clear_error();
    ALCH_TRY(check_shape(shape));
    ALCH_TRY(check_batch(batch));
    ALCH_TRY(check_saved_weights(saved, weights, batch->total_tokens));
    ALCH_TRY(check_wgrads(wgrads));
    REQUIRE_ACT(dY, "dY", batch->total_tokens);
    REQUIRE_ACT(dX, "dX", batch->total_tokens);
    const size_t need = plan_layer_bwd(*shape, batch->total_tokens, nullptr, 0).bytes;
    if (!workspace || workspace_bytes < need) return fail(ALCH_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", workspace_bytes, need);
    if (!aligned16(workspace)) return fail(ALCH_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    const LayerBwdPlan p = plan_layer_bwd(*shape, batch->total_tokens, workspace, workspace_bytes);
    return layer_backward_enqueue(*shape, *batch, *saved, *weights, dY, loss_mask, dX, wgrads, p,
                                  static_cast<hipStream_t>(hip_stream));
}

static int check_lora(const alch_layer_shape* s, const alch_lora* lora, const alch_lora_grads* lg) {
    if (!lora) return fail(ALCH_ERR_INVALID_ARG, "lora is NULL");
    if (lora->rank < 8 || lora->rank > kLoraSlot || lora->rank % 8)
        return fail(ALCH_ERR_SHAPE, "adapter rank %d: must be a multiple of 8 in 8..%d", lora->rank, kLoraSlot);
    const int QD = s->n_q_heads * s->head_dim, KD = s->n_kv_heads * s->head_dim;
    if (s->hidden % 8 || s->ffn % 8 || QD % 8 || KD % 8)
        return fail(ALCH_ERR_UNSUPPORTED, "adapters need every projection width to be a multiple of 8");
    for (int p = 0; p < ALCH_N_PROJ; ++p) {
        if ((lora->A[p] == nullptr) != (lora->B[p] == nullptr))
            return fail(ALCH_ERR_INVALID_ARG, "adapter %d: A and B must both be given or both be NULL", p);
        if (!aligned16(lora->A[p]) || !aligned16(lora->B[p]))
            return fail(ALCH_ERR_INVALID_ARG, "adapter %d: A or B is not 16-byte aligned", p);
        if (lg) {
            if ((lg->dA[p] || lg->dB[p]) && !lora->A[p])
                return fail(ALCH_ERR_INVALID_ARG, "adapter %d: gradient requested for a projection without adapter", p);
            if (!aligned16(lg->dA[p]) || !aligned16(lg->dB[p]))
                return fail(ALCH_ERR_INVALID_ARG, "adapter %d: dA or dB is not 16-byte aligned", p);
        }
    }
    return ALCH_OK;
}

size_t alch_layer_backward_lora_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens, int32_t max_seqlen,
                                                int32_t rank) {
    (void)max_seqlen;
    if (!shape || check_shape(shape) != ALCH_OK || total_tokens < 0 || rank < 8 || rank > kLoraSlot || rank % 8) return 0;
    return plan_layer_bwd(*shape, total_tokens, nullptr, 0, rank).bytes;
}

int alch_layer_backward_lora(const alch_layer_shape* shape, const alch_batch* batch, const alch_saved* saved,
                             const alch_weights* weights, const alch_lora* lora, const void* dY,
                             const uint8_t* loss_mask, void* dX, const alch_wgrads* wgrads,
                             const alch_lora_grads* lora_grads, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
    clear_error();
    ALCH_TRY(check_shape(shape));
    ALCH_TRY(check_batch(batch));
    ALCH_TRY(check_saved_weights(saved, weights, batch->total_tokens));
    ALCH_TRY(check_wgrads(wgrads));
    ALCH_TRY(check_lora(shape, lora, lora_grads));
    REQUIRE_ACT(dY, "dY", batch->total_tokens);
    REQUIRE_ACT(dX, "dX", batch->total_tokens);
    const size_t need = plan_layer_bwd(*shape, batch->total_tokens, nullptr, 0, lora->rank).bytes;
    if (!workspace || workspace_bytes < need) return fail(ALCH_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", workspace_bytes, need);
    if (!aligned16(workspace)) return fail(ALCH_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    const LayerBwdPlan p = plan_layer_bwd(*shape, batch->total_tokens, workspace, workspace_bytes, lora->rank);
    return layer_backward_enqueue(*shape, *batch, *saved, *weights, dY, loss_mask, dX, wgrads, p,
                                  static_cast<hipStream_t>(hip_stream), lora, lora_grads);
}

size_t alch_stack_backward_workspace_bytes(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                                           int32_t total_tokens, int32_t max_seqlen) {
    (void)max_seqlen; (void)n_layers;
    if (!shape || check_shape(shape) != ALCH_OK || total_tokens < 0 || vocab <= 0) return 0;
    return plan_stack(*shape, vocab, total_tokens, nullptr, 0).bytes;
}

// The head is cross-entropy on `labels` (dpo == nullptr) or DPO on the scored items of `dpo`.
static int stack_backward_impl(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab, const alch_batch* batch,
                               const alch_saved* saved, const alch_weights* weights, const alch_lora* lora,
                               const void* X_final, const void* g_final, const void* W_lm, const int32_t* labels,
                               const uint8_t* loss_mask, const alch_wgrads* wgrads, const alch_lora_grads* lora_grads,
                               void* dg_final, void* dW_lm, void* dX_embed, float* loss_out, const alch_hooks* hooks,
                               void* workspace, size_t workspace_bytes, void* hip_stream, const alch_dpo* dpo = nullptr) {
    clear_error();
    ALCH_TRY(check_shape(shape));
    ALCH_TRY(check_batch(batch));
    if (n_layers < 0) return fail(ALCH_ERR_INVALID_ARG, "n_layers < 0");
    if (vocab <= 0) return fail(ALCH_ERR_SHAPE, "vocab <= 0");
    if (n_layers > 0 && (!saved || !weights)) return fail(ALCH_ERR_INVALID_ARG, "saved / weights array is NULL");
    for (int l = 0; l < n_layers; ++l) {
        ALCH_TRY(check_saved_weights(&saved[l], &weights[l], batch->total_tokens));
        if (wgrads) ALCH_TRY(check_wgrads(&wgrads[l]));
        if (lora) {
            ALCH_TRY(check_lora(shape, &lora[l], lora_grads ? &lora_grads[l] : nullptr));
            if (lora[l].rank != lora[0].rank) return fail(ALCH_ERR_SHAPE, "layer %d: adapter rank differs from layer 0", l);
        }
    }
    const int rank = (lora && n_layers > 0) ? lora[0].rank : 0;
    REQUIRE_ACT(X_final, "X_final", batch->total_tokens); REQUIRE_PTR(g_final, "g_final"); REQUIRE_PTR(W_lm, "W_lm");
    REQUIRE_ACT(dX_embed, "dX_embed", batch->total_tokens);
    if ((!dpo && batch->total_tokens > 0 && !labels) || !loss_out) return fail(ALCH_ERR_INVALID_ARG, "labels / loss_out is NULL");
    OPTIONAL_PTR(dg_final, "dg_final"); OPTIONAL_PTR(dW_lm, "dW_lm");
    if (dpo) {
        if (dpo->n_items < 0 || dpo->n_pairs < 0) return fail(ALCH_ERR_INVALID_ARG, "dpo: negative n_items / n_pairs");
        if (dpo->n_items > batch->total_tokens) return fail(ALCH_ERR_SHAPE, "dpo: %d items > %d tokens", dpo->n_items, batch->total_tokens);
        if (2 * (long long)dpo->n_pairs > batch->total_tokens) return fail(ALCH_ERR_SHAPE, "dpo: %d pairs need more slots than there are tokens", dpo->n_pairs);
        if (dpo->n_items > 0 && (!dpo->item_row || !dpo->item_label || !dpo->item_slot || !dpo->item_row_host))
            return fail(ALCH_ERR_INVALID_ARG, "dpo: item_row / item_label / item_slot / item_row_host is NULL");
        if (dpo->n_pairs > 0 && !dpo->ref_logp) return fail(ALCH_ERR_INVALID_ARG, "dpo: ref_logp is NULL");
        if (((size_t)shape->hidden * dtype_size(shape->dtype)) % 16)
            return fail(ALCH_ERR_UNSUPPORTED, "dpo: a hidden row of %d elements is not a multiple of 16 bytes", shape->hidden);
        for (int m = 0; m < dpo->n_items; ++m) {
            const int r = dpo->item_row_host[m];
            if (r < 0 || r >= batch->total_tokens) return fail(ALCH_ERR_SHAPE, "dpo: item_row[%d] = %d outside the batch", m, r);
            if (m > 0 && r < dpo->item_row_host[m - 1]) return fail(ALCH_ERR_SHAPE, "dpo: item_row is not ascending at item %d", m);
        }
    }
    const size_t need = plan_stack(*shape, vocab, batch->total_tokens, nullptr, 0, rank).bytes;
    if (!workspace || workspace_bytes < need) return fail(ALCH_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", workspace_bytes, need);
    if (!aligned16(workspace)) return fail(ALCH_ERR_INVALID_ARG, "workspace is not 16-byte aligned");

    const alch_layer_shape& s = *shape;
    const StackPlan p = plan_stack(s, vocab, batch->total_tokens, workspace, workspace_bytes, rank);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const alch_dtype dt = s.dtype;
    const size_t E = dtype_size(dt);
    const int T = batch->total_tokens, H = s.hidden;
    const int acc = wgrads ? (wgrads[0].accumulate != 0) : 0;
    // scratch of split products in the head: the layers' workspace, idle until the walk starts
    auto gemm_ws = [&](alch_dtype t, int M, int N, bool a_k, bool b_k) {
        GemmDesc d = gemm(t, M, N, a_k, b_k);
        d.split_ws = p.layer_ws;
        d.split_ws_bytes = p.layer_ws_bytes;
        return d;
    };

    bool compact_head = false;
    if (dpo) {
        // DPO head: the stack-output rows of the scored tokens are gathered into [n_items, H]; pass 1 turns each
        // chunk of their logits into log-probabilities, the slot sums give z, the loss and a weight per slot;
        // pass 2 forms the logits gradient (recomputing the logits unless one chunk holds them all) and the two
        // products; the row gradients are summed back into a zero-filled [T, H] (a row may score several tokens).
        const int M = dpo->n_items, n_slots = 2 * dpo->n_pairs;
        ALCH_TRY(launch_rmsnorm_fwd(dt, X_final, g_final, p.Hf, T, H, s.rms_eps, st));
        if (M > 0) ALCH_TRY(launch_scatter_rows(p.Hf, dpo->item_row, p.h_Hf, M, (size_t)H * E, st));  // h_Hf[m] = Hf[item_row[m]]
        const bool one_chunk = M <= kHeadChunkRows;
        auto logits_of = [&](int r0, int rows) {
            GemmDesc d = gemm_ws(dt, rows, vocab, true, true);
            add_seg(d, at(p.h_Hf, (size_t)r0 * H, E), H, W_lm, H, H);
            add_out(d, p.logits, 0, vocab);
            return launch_gemm(d, st);
        };
        for (int r0 = 0; r0 < M; r0 += kHeadChunkRows) {
            const int rows = M - r0 < kHeadChunkRows ? M - r0 : kHeadChunkRows;
            ALCH_TRY(logits_of(r0, rows));
            ALCH_TRY(launch_dpo_logp(dt, p.logits, vocab, rows, vocab, dpo->item_label + r0, p.dpo_logp + r0, p.dpo_logz + r0, st));
        }
        ALCH_TRY(launch_dpo_weights(p.dpo_logp, dpo->item_slot, dpo->item_label, M, vocab, dpo->ref_logp, dpo->n_pairs,
                                    dpo->beta, p.dpo_pi, p.dpo_w, dpo->z_out, loss_out, st));
        bool first = true;
        for (int r0 = 0; r0 < M; r0 += kHeadChunkRows) {
            const int rows = M - r0 < kHeadChunkRows ? M - r0 : kHeadChunkRows;
            if (!one_chunk) ALCH_TRY(logits_of(r0, rows));
            ALCH_TRY(launch_dpo_grad(dt, p.logits, vocab, rows, vocab, dpo->item_label + r0, dpo->item_slot + r0,
                                     p.dpo_logz + r0, p.dpo_w, n_slots, st));
            {  // gradient of the gathered rows = dlogits W_lm
                GemmDesc d = gemm_ws(dt, rows, H, true, false);
                add_seg(d, p.logits, vocab, W_lm, H, vocab);
                add_out(d, at(p.h_dHf, (size_t)r0 * H, E), 0, H);
                ALCH_TRY(launch_gemm(d, st));
            }
            if (dW_lm) {  // dW_lm (+)= dlogits^T Hf
                GemmDesc d = gemm_ws(dt, vocab, H, false, false);
                add_seg(d, p.logits, vocab, at(p.h_Hf, (size_t)r0 * H, E), H, rows);
                add_out(d, dW_lm, 0, H);
                d.accumulate = first ? acc : 1;
                ALCH_TRY(launch_gemm(d, st));
            }
            first = false;
        }
        if (M == 0 && dW_lm && !acc) {
            GemmDesc d = gemm_ws(dt, vocab, H, false, false);  // zero rows contracted: writes zeros
            add_seg(d, p.logits, vocab, p.Hf, H, 0);
            add_out(d, dW_lm, 0, H);
            ALCH_TRY(launch_gemm_generic(d, st));
        }
        ALCH_TRY(launch_dpo_scatter(dt, p.h_dHf, dpo->item_row, M, p.dHf, T, H, st));
    } else {
        // LM head + cross-entropy in row chunks: logits -> dlogits in place, never stored whole.
        // With a loss mask (bf16, matrix-core shapes) only the counted tokens -- label >= 0 and mask byte nonzero --
        // go through the head: their Hf rows and labels are gathered, the three products and the cross-entropy
        // take their row counts from device memory, and dHf is scattered back into a zero-filled [T, H].
        compact_head = loss_mask && T > 0 && dt == ALCH_BF16 && H % 64 == 0 && vocab % 64 == 0 &&
                       (long long)kHeadChunkRows * vocab * (long long)E < (1LL << 31);
        ALCH_TRY(launch_count_labels(labels, loss_mask, T, vocab, p.n_counted, p.row_loss, st));
        ALCH_TRY(launch_rmsnorm_fwd(dt, X_final, g_final, p.Hf, T, H, s.rms_eps, st));
        const void* head_in = p.Hf;
        void* head_out = p.dHf;
        const int* head_labels = labels;
        const uint8_t* head_mask = loss_mask;
        if (compact_head) {
            ALCH_TRY(launch_counted_mask(labels, loss_mask, T, vocab, p.h_counted, st));
            const alch_stream rows1[1] = {{p.Hf, p.h_Hf, (size_t)H * E, (size_t)H * E}};
            ALCH_TRY(launch_pack(p.h_counted, T, batch->cu_seqlens, 0, 1, rows1, T, p.h_index, p.h_cu, p.h_n, p.h_packws, st, false));
            ALCH_TRY(launch_gather_int(labels, p.h_index, p.h_n, p.h_labels, T, st));
            ALCH_TRY(launch_rank_of_kept(p.h_index, p.h_n, p.h_inv, T, st));
            ALCH_TRY(launch_chunk_rows(p.h_n, ceil_div(T, kHeadChunkRows), kHeadChunkRows, p.h_chunk_rows, st));
            head_in = p.h_Hf; head_out = p.h_dHf; head_labels = p.h_labels; head_mask = nullptr;
        }
        bool first = true;
        for (int r0 = 0; r0 < T; r0 += kHeadChunkRows) {
            const int rows = T - r0 < kHeadChunkRows ? T - r0 : kHeadChunkRows;
            const int* rows_dev = compact_head ? p.h_chunk_rows + r0 / kHeadChunkRows : nullptr;
            const void* hf = at(head_in, (size_t)r0 * H, E);
            {  // logits = Hf W_lm^T
                GemmDesc d = gemm_ws(dt, rows, vocab, true, true);
                add_seg(d, hf, H, W_lm, H, H);
                add_out(d, p.logits, 0, vocab);
                d.m_dev = rows_dev;
                ALCH_TRY(launch_gemm(d, st));
            }
            ALCH_TRY(launch_ce_chunk(dt, p.logits, vocab, rows, vocab, head_labels + r0, head_mask ? head_mask + r0 : nullptr,
                                     p.n_counted, p.row_loss + r0, st, rows_dev));
            {  // dHf = dlogits W_lm
                GemmDesc d = gemm_ws(dt, rows, H, true, false);
                add_seg(d, p.logits, vocab, W_lm, H, vocab);
                add_out(d, const_cast<char*>(at(head_out, (size_t)r0 * H, E)), 0, H);
                d.m_dev = rows_dev;
                ALCH_TRY(launch_gemm(d, st));
            }
            if (dW_lm) {  // dW_lm (+)= dlogits^T Hf
                GemmDesc d = gemm_ws(dt, vocab, H, false, false);
                add_seg(d, p.logits, vocab, hf, H, rows);
                add_out(d, dW_lm, 0, H);
                d.accumulate = first ? acc : 1;
                d.k_dev = rows_dev;
                ALCH_TRY(launch_gemm(d, st));
            }
            first = false;
        }
        if (compact_head) ALCH_TRY(launch_scatter_rows(p.h_dHf, p.h_inv, p.dHf, T, (size_t)H * E, st));
        if (T == 0 && dW_lm && !acc) {
            GemmDesc d = gemm_ws(dt, vocab, H, false, false);  // zero rows contracted: writes zeros
            add_seg(d, p.logits, vocab, p.Hf, H, 0);
            add_out(d, dW_lm, 0, H);
            ALCH_TRY(launch_gemm_generic(d, st));
        }
        ALCH_TRY(launch_finish_loss(p.row_loss, p.n_counted, loss_out, T, st));

    }

    // final RMSNorm backward -> gradient w.r.t. the last layer's output
    void* cur = n_layers == 0 ? dX_embed : p.ping;
    ALCH_TRY(launch_rmsnorm_bwd(dt, p.dHf, X_final, g_final, nullptr, nullptr, cur, dg_final, acc, p.partial, T, H,
                                s.rms_eps, st));

    const LayerBwdPlan lp = plan_layer_bwd(s, T, p.layer_ws, p.layer_ws_bytes, rank);
    for (int l = n_layers - 1; l >= 0; --l) {
        if (hooks && hooks->preempt && hooks->preempt(hooks->user, l) != 0)
            return fail(ALCH_ERR_ABORTED, "preempt hook stopped the walk before layer %d", l);
        if (hooks && hooks->layer_ready && hooks->layer_ready(hooks->user, l) != 0)
            return fail(ALCH_ERR_ABORTED, "layer_ready hook failed for layer %d", l);
        void* out = l == 0 ? dX_embed : (cur == p.ping ? p.pong : p.ping);
        // the gradient entering the top layer is exactly zero in the rows the head did not count: that layer may
        // compact its row-local part (lower layers see dense gradients: attention spreads them over earlier tokens)
        const uint8_t* top_mask = (compact_head && l == n_layers - 1) ? p.h_counted : nullptr;
        ALCH_TRY(layer_backward_enqueue(s, *batch, saved[l], weights[l], cur, top_mask, out,
                                        wgrads ? &wgrads[l] : nullptr, lp, st, lora ? &lora[l] : nullptr,
                                        lora_grads ? &lora_grads[l] : nullptr));
        cur = out;
    }
    return ALCH_OK;
}

int alch_stack_backward(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab, const alch_batch* batch,
                        const alch_saved* saved, const alch_weights* weights, const void* X_final,
                        const void* g_final, const void* W_lm, const int32_t* labels, const uint8_t* loss_mask,
                        const alch_wgrads* wgrads, void* dg_final, void* dW_lm, void* dX_embed, float* loss_out,
                        const alch_hooks* hooks, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return stack_backward_impl(shape, n_layers, vocab, batch, saved, weights, nullptr, X_final, g_final, W_lm, labels,
                               loss_mask, wgrads, nullptr, dg_final, dW_lm, dX_embed, loss_out, hooks, workspace,
                               workspace_bytes, hip_stream);
}

size_t alch_stack_backward_lora_workspace_bytes(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                                                int32_t total_tokens, int32_t max_seqlen, int32_t rank) {
    (void)max_seqlen; (void)n_layers;
    if (!shape || check_shape(shape) != ALCH_OK || total_tokens < 0 || vocab <= 0 || rank < 8 || rank > kLoraSlot || rank % 8)
        return 0;
    return plan_stack(*shape, vocab, total_tokens, nullptr, 0, rank).bytes;
}

int alch_stack_backward_lora(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab, const alch_batch* batch,
                             const alch_saved* saved, const alch_weights* weights, const alch_lora* lora,
                             const void* X_final, const void* g_final, const void* W_lm, const int32_t* labels,
                             const uint8_t* loss_mask, const alch_wgrads* wgrads, const alch_lora_grads* lora_grads,
                             void* dg_final, void* dW_lm, void* dX_embed, float* loss_out, const alch_hooks* hooks,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n_layers > 0 && !lora) {
        clear_error();
        return fail(ALCH_ERR_INVALID_ARG, "lora array is NULL");
    }
    return stack_backward_impl(shape, n_layers, vocab, batch, saved, weights, lora, X_final, g_final, W_lm, labels,
                               loss_mask, wgrads, lora_grads, dg_final, dW_lm, dX_embed, loss_out, hooks, workspace,
                               workspace_bytes, hip_stream);
}

int alch_stack_backward_dpo(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab, const alch_batch* batch,
                            const alch_saved* saved, const alch_weights* weights, const alch_lora* lora,
                            const void* X_final, const void* g_final, const void* W_lm, const alch_dpo* dpo,
                            const alch_wgrads* wgrads, const alch_lora_grads* lora_grads, void* dg_final, void* dW_lm,
                            void* dX_embed, float* loss_out, const alch_hooks* hooks, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
    if (!dpo) {
        clear_error();
        return fail(ALCH_ERR_INVALID_ARG, "dpo is NULL");
    }
    return stack_backward_impl(shape, n_layers, vocab, batch, saved, weights, lora, X_final, g_final, W_lm, nullptr,
                               nullptr, wgrads, lora ? lora_grads : nullptr, dg_final, dW_lm, dX_embed, loss_out, hooks,
                               workspace, workspace_bytes, hip_stream, dpo);
}

int alch_attention_forward(const alch_layer_shape* shape, const alch_batch* batch, const void* Q, const void* K,
                           const void* V, void* O, float* LSE, void* hip_stream) {
    clear_error();
    ALCH_TRY(check_shape(shape));
    ALCH_TRY(check_batch(batch));
    const int T = batch->total_tokens;
    REQUIRE_ACT(Q, "Q", T); REQUIRE_ACT(K, "K", T); REQUIRE_ACT(V, "V", T); REQUIRE_ACT(O, "O", T);
    REQUIRE_ACT(LSE, "LSE", T);
    return launch_attn_fwd(shape->dtype, Q, K, V, O, LSE, T, batch->n_seqs, batch->max_seqlen, batch->cu_seqlens,
                           batch->cu_seqlens_host, batch->seq_prefix, batch->seq_prefix_host, 0, shape->n_q_heads,
                           shape->n_kv_heads, shape->head_dim, static_cast<hipStream_t>(hip_stream));
}

size_t alch_layer_forward_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens, int32_t max_seqlen) {
    (void)max_seqlen;
    if (!shape || check_shape(shape) != ALCH_OK || total_tokens < 0) return 0;
    return plan_layer_fwd(*shape, total_tokens, nullptr, 0).bytes;
}

// Forward of sequences seq_begin .. n_seqs-1 (rows r0 = cu[seq_begin] .. T-1 of every tensor); arguments validated.
static int layer_forward_impl(const alch_layer_shape* shape, const alch_batch* batch, int seq_begin, const void* X,
                              const alch_weights* w, void* Y, const alch_record_out* rec, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
    ALCH_TRY(check_shape(shape));
    ALCH_TRY(check_batch(batch));
    if (seq_begin < 0 || seq_begin > batch->n_seqs) return fail(ALCH_ERR_INVALID_ARG, "seq_begin %d outside 0..n_seqs", seq_begin);
    if (seq_begin > 0 && batch->total_tokens > 0 && !batch->positions)
        return fail(ALCH_ERR_INVALID_ARG, "positions must be given with seq_begin > 0");
    if (!w || !rec) return fail(ALCH_ERR_INVALID_ARG, "weights / record_out is NULL");
    REQUIRE_PTR(X, "X"); REQUIRE_PTR(Y, "Y");
    REQUIRE_PTR(w->Wq, "weights.Wq"); REQUIRE_PTR(w->Wk, "weights.Wk"); REQUIRE_PTR(w->Wv, "weights.Wv");
    REQUIRE_PTR(w->Wo, "weights.Wo"); REQUIRE_PTR(w->Wg, "weights.Wg"); REQUIRE_PTR(w->Wu, "weights.Wu");
    REQUIRE_PTR(w->Wd, "weights.Wd"); REQUIRE_PTR(w->g1, "weights.g1"); REQUIRE_PTR(w->g2, "weights.g2");
    REQUIRE_PTR(rec->X, "record_out.X"); REQUIRE_PTR(rec->X2, "record_out.X2"); REQUIRE_PTR(rec->Q, "record_out.Q");
    REQUIRE_PTR(rec->K, "record_out.K"); REQUIRE_PTR(rec->V, "record_out.V"); REQUIRE_PTR(rec->O, "record_out.O");
    REQUIRE_PTR(rec->G, "record_out.G"); REQUIRE_PTR(rec->U, "record_out.U"); REQUIRE_PTR(rec->LSE, "record_out.LSE");
    const int r0 = batch->cu_seqlens_host[seq_begin];
    const int T = batch->total_tokens - r0;  // rows computed
    const size_t need = plan_layer_fwd(*shape, T, nullptr, 0).bytes;
    if (!workspace || workspace_bytes < need) return fail(ALCH_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", workspace_bytes, need);
    if (!aligned16(workspace)) return fail(ALCH_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    if (T <= 0) return ALCH_OK;

    const alch_layer_shape& s = *shape;
    const LayerFwdPlan p = plan_layer_fwd(s, T, workspace, workspace_bytes);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const alch_dtype dt = s.dtype;
    const size_t E = dtype_size(dt);
    const int H = s.hidden, F = s.ffn, D = s.head_dim;
    const int QD = s.n_q_heads * D, KD = s.n_kv_heads * D;
    auto gemm_ws = [&](alch_dtype t, int M, int N, bool a_k, bool b_k) {
        GemmDesc d = gemm(t, M, N, a_k, b_k);
        d.split_ws = p.gemm_ws;
        d.split_ws_bytes = kGemmSplitWsBytes;
        return d;
    };
    // the computed rows of every [total_tokens, width] tensor
    const void* Xr = at(X, (size_t)r0 * H, E);
    void* Yr = at(Y, (size_t)r0 * H, E);
    void *rX = at(rec->X, (size_t)r0 * H, E), *rX2 = at(rec->X2, (size_t)r0 * H, E), *rQ = at(rec->Q, (size_t)r0 * QD, E);
    void *rK = at(rec->K, (size_t)r0 * KD, E), *rV = at(rec->V, (size_t)r0 * KD, E);
    void *rG = at(rec->G, (size_t)r0 * F, E), *rU = at(rec->U, (size_t)r0 * F, E), *rO = at(rec->O, (size_t)r0 * QD, E);
    // positions follow the rows; without them (seq_begin = 0 only) the kernels count inside each sequence
    const int* pos = batch->positions ? batch->positions + r0 : nullptr;

    if (rX != Xr) ALCH_TRY(launch_masked_copy(dt, Xr, nullptr, rX, T, H, st));
    ALCH_TRY(launch_rmsnorm_fwd(dt, Xr, w->g1, p.Hn, T, H, s.rms_eps, st));
    const void* Ws[3] = {w->Wq, w->Wk, w->Wv};
    void* outs[3] = {rQ, rK, rV};
    const int widths[3] = {QD, KD, KD};
    for (int i = 0; i < 3; ++i) {
        GemmDesc d = gemm_ws(dt, T, widths[i], true, true);
        add_seg(d, p.Hn, H, Ws[i], H, H);
        add_out(d, outs[i], 0, widths[i]);
        ALCH_TRY(launch_gemm(d, st));
    }
    ALCH_TRY(launch_rope(dt, rQ, QD, T, s.n_q_heads, D, pos, batch->cu_seqlens, batch->n_seqs, s.rope_base, 1.f, st));
    ALCH_TRY(launch_rope(dt, rK, KD, T, s.n_kv_heads, D, pos, batch->cu_seqlens, batch->n_seqs, s.rope_base, 1.f, st));
    // attention indexes whole-batch rows: the keys and values of a prefix sequence lie before r0
    ALCH_TRY(launch_attn_fwd(dt, rec->Q, rec->K, rec->V, rec->O, rec->LSE, batch->total_tokens, batch->n_seqs,
                             batch->max_seqlen, batch->cu_seqlens, batch->cu_seqlens_host, batch->seq_prefix,
                             batch->seq_prefix_host, seq_begin, s.n_q_heads, s.n_kv_heads, D, st));
    {  // X2 = X + O Wo^T
        ALCH_TRY(launch_masked_copy(dt, Xr, nullptr, rX2, T, H, st));
        GemmDesc d = gemm_ws(dt, T, H, true, true);
        add_seg(d, rO, QD, w->Wo, QD, QD);
        add_out(d, rX2, 0, H);
        d.accumulate = 1;
        ALCH_TRY(launch_gemm(d, st));
    }
    ALCH_TRY(launch_rmsnorm_fwd(dt, rX2, w->g2, p.Hn, T, H, s.rms_eps, st));
    const void* Wm[2] = {w->Wg, w->Wu};
    void* om[2] = {rG, rU};
    for (int i = 0; i < 2; ++i) {
        GemmDesc d = gemm_ws(dt, T, F, true, true);
        add_seg(d, p.Hn, H, Wm[i], H, H);
        add_out(d, om[i], 0, F);
        ALCH_TRY(launch_gemm(d, st));
    }
    ALCH_TRY(launch_swiglu_act(dt, rG, rU, p.Act, (long long)T * F, st));
    {  // Y = X2 + Act Wd^T
        ALCH_TRY(launch_masked_copy(dt, rX2, nullptr, Yr, T, H, st));
        GemmDesc d = gemm_ws(dt, T, H, true, true);
        add_seg(d, p.Act, F, w->Wd, F, F);
        add_out(d, Yr, 0, H);
        d.accumulate = 1;
        ALCH_TRY(launch_gemm(d, st));
    }
    return ALCH_OK;
}

int alch_layer_forward(const alch_layer_shape* shape, const alch_batch* batch, const void* X,
                       const alch_weights* w, void* Y, const alch_record_out* rec, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
    clear_error();
    return layer_forward_impl(shape, batch, 0, X, w, Y, rec, workspace, workspace_bytes, hip_stream);
}

int alch_layer_forward_from(const alch_layer_shape* shape, const alch_batch* batch, int32_t seq_begin, const void* X,
                            const alch_weights* w, void* Y, const alch_record_out* rec, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
    clear_error();
    return layer_forward_impl(shape, batch, seq_begin, X, w, Y, rec, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
