// Internal launch interfaces between the translation units of libalch.
#pragma once
#include "common.h"

namespace alch {

// ---- capture/pack ----------------------------------------------------------------------
static constexpr int kMaxStreamsPerLaunch = 16;
static constexpr int kGatherGridMax = 1 << 20;  // one work-group per candidate row, capped
size_t pack_workspace_bytes(int total_tokens);
int launch_pack(const uint8_t* mask, int T, const int* cu_seqlens, int n_seqs, int n_streams,
                const alch_stream* streams, long long capacity, int* kept_index, int* cu_kept,
                int* n_kept_and_status, void* workspace, hipStream_t stream, bool traced = true);
int launch_pack_gather(int T, int n_streams, const alch_stream* streams, long long capacity, const int* kept_index,
                       const int* n_kept_and_status, hipStream_t stream, bool traced = true);

// ---- GEMM ------------------------------------------------------------------------------
// C[M,N] (+)= sum over segments of A_s(M,K_s) * B_s(K_s,N), fp32 accumulation.
//   a_kmajor: A(m,k) = A[m*lda + k]   else A(m,k) = A[k*lda + m]
//   b_kmajor: B(k,n) = B[n*ldb + k]   else B(k,n) = B[k*ldb + n]
// The output may be split along M into up to three row ranges with their own base
// pointers (rows [m_begin_i, m_begin_{i+1}) go to out[i].C, row index relative to
// m_begin_i, leading dimension ldc).
static constexpr int kMaxGemmSegs = 4;  // operand pairs summed into one product
static constexpr int kMaxGemmOuts = 3;  // row ranges of C with their own base pointers
struct GemmSeg {
    const void* A;
    const void* B;
    int K;
    long long lda, ldb;
};
struct GemmOut {
    void* C;
    int m_begin;
    long long ldc;
};
enum GemmEpilogue { kEpiNone = 0, kEpiSwigluBwd = 1 };
struct GemmDesc {
    int M = 0, N = 0;
    bool a_kmajor = true, b_kmajor = true;
    int n_seg = 0;
    GemmSeg seg[kMaxGemmSegs];
    int n_out = 0;
    GemmOut out[kMaxGemmOuts];
    int accumulate = 0;
    alch_dtype dtype = ALCH_BF16;
    // kEpiSwigluBwd: the product is dAct [M, N]; with G, U [M, N] (ld = ldgu) the kernel writes
    // dG to out[0].C[:, 0:N], dU to out[0].C[:, N:2N] and Act = silu(G)*U to act_out [M, N].
    int epilogue = kEpiNone;
    const void* G = nullptr;
    const void* U = nullptr;
    long long ldgu = 0;
    void* act_out = nullptr;
    const uint8_t* row_mask = nullptr;  // optional: rows of A whose mask byte is 0 count as zero (A k-major only)
    // optional device-resident sizes (matrix-core kernel only): effective M = min(*m_dev, M); effective K of
    // every operand pair = min(*k_dev, K).  Rows / contraction steps beyond them are neither read nor written.
    const int* m_dev = nullptr;
    const int* k_dev = nullptr;
    // optional scratch (matrix-core kernel only): when the last round of tiles would leave at least half of the
    // compute units idle, every tile of that round is split along the contraction over s work-groups, which
    // write fp32 partial tiles here; a second kernel adds them in a fixed order.  kGemmSplitWsBytes always suffices.
    void* split_ws = nullptr;
    size_t split_ws_bytes = 0;
};
static constexpr size_t kGemmSplitWsBytes = (size_t)64 << 20;
int launch_gemm(const GemmDesc& d, hipStream_t stream);
// used by launch_gemm
bool gemm_mfma_supported(const GemmDesc& d);
int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream);
int launch_gemm_generic(const GemmDesc& d, hipStream_t stream);

// ---- row-wise kernels --------------------------------------------------------------------
// H = X * rsqrt(mean(X^2)+eps) * g   (rows of width `width`)
// rows_dev (optional, bf16 row kernel only): the row count is min(*rows_dev, T), read on the device.
int launch_rmsnorm_fwd(alch_dtype dt, const void* X, const void* g, void* H, int T, int width, float eps,
                       hipStream_t stream, const int* rows_dev = nullptr);
// dX = resid + rmsnorm_bwd(dH; X, g)   (resid may be NULL; resid_mask zeroes resid rows where mask==0);
// dg (+)= sum_t dH*X*r  (dg may be NULL).  partial: fp32 scratch [rmsnorm_bwd_blocks(T), width].
// hn_out (may be NULL): also writes the normalised rows X*r*g themselves, the operand of the weight gradients
// that follow, so that X is read once for both.
int rmsnorm_bwd_blocks(int T);
int launch_rmsnorm_bwd(alch_dtype dt, const void* dH, const void* X, const void* g, const void* resid,
                       const uint8_t* resid_mask, void* dX, void* dg, int accumulate, float* partial, int T,
                       int width, float eps, hipStream_t stream, const int* rows_dev = nullptr, void* hn_out = nullptr);
// inv[t] = rank of token t among the first *n_rows entries of index (the kept tokens), -1 if absent
int launch_rank_of_kept(const int* index, const int* n_rows, int* inv, int T, hipStream_t stream);
// out [T, row_bytes] = src[inv[t], :] where inv[t] >= 0, zeros elsewhere
int launch_scatter_rows(const void* src, const int* inv, void* out, int T, size_t row_bytes, hipStream_t stream);
// Act = silu(G) * U
int launch_swiglu_act(alch_dtype dt, const void* G, const void* U, void* Act, long long n, hipStream_t stream);
// dGU[:, 0:F] = dAct*U*silu'(G), dGU[:, F:2F] = dAct*silu(G); optionally Act = silu(G)*U
int launch_swiglu_bwd(alch_dtype dt, const void* dAct, const void* G, const void* U, void* dGU, void* Act,
                      int T, int F, hipStream_t stream);
// delta[t,h] = sum_d dO[t,h,d] * O[t,h,d]   (fp32 out)
int launch_attn_delta(alch_dtype dt, const void* dO, const void* O, float* delta, int T, int Hq, int D,
                      hipStream_t stream);
// In-place rotary rotation of x [T, n_heads, D] (row stride ld elements) by sign * angle.
int launch_rope(alch_dtype dt, void* x, long long ld, int T, int n_heads, int D, const int* positions,
                const int* cu_seqlens, int n_seqs, float base, float sign, hipStream_t stream);
// out = a with rows zeroed where mask == 0 (mask may be NULL: plain copy)
int launch_masked_copy(alch_dtype dt, const void* a, const uint8_t* mask, void* out, int T, int width,
                       hipStream_t stream);
// y = a + b
int launch_add(alch_dtype dt, const void* a, const void* b, void* y, long long n, hipStream_t stream);

// ---- low-rank adapters ---------------------------------------------------------------------
static constexpr int kLoraSlot = 64;       // columns of one zero-padded rank slot (rank <= 64)
static constexpr int kLoraMaxSplits = 64;  // token splits of the adapter-gradient reduction
// Y[t, 0:r] = alpha * sum_k X[t, k] * S[j*lds + k] (S is an [r, K] matrix); columns r .. slot_cols-1 of Y
// are written as zeros; r = 0 (S may be null) zero-fills the slot.  Up to three problems per launch, all
// with Trows rows, the same alpha, and outputs of row stride ldy.
struct LoraDown {
    const void* X; long long ldx; int K;
    const void* S; long long lds; int r;
    void* Y;
};
int launch_lora_down(alch_dtype dt, const LoraDown* jobs, int n_jobs, int Trows, float alpha, long long ldy,
                     int slot_cols, hipStream_t stream);
// C(j, n) (+)= alpha * sum_t S[t*lds + j] * X[t*ldx + n], j < r, n < N; stored C[j*ldc + n], or C[n*ldc + j]
// when transposed.  Up to kLoraUpJobs problems per launch pair, all with Trows rows, the same r, alpha and
// accumulate.  scratch: lora_up_scratch_bytes(r, sum of the N of the jobs) bytes of fp32 partial sums.
static constexpr int kLoraUpJobs = 6;
struct LoraUp {
    const void* S; long long lds;
    const void* X; long long ldx;
    int N;
    void* C; long long ldc;
    int transposed;
};
size_t lora_up_scratch_bytes(int rank, int n_sum);
int launch_lora_up(alch_dtype dt, const LoraUp* jobs, int n_jobs, int Trows, int r, float alpha, int accumulate,
                   float* scratch, hipStream_t stream);
// Operand preparation: job i writes dst [rows_out, cols] = src [r, cols] (or, transpose, src [cols, r]
// transposed) followed by zero rows; src null: all zeros.
struct LoraPrepJob {
    const void* src; void* dst;
    int r, cols, rows_out, transpose;
};
struct LoraPrepParams { LoraPrepJob job[16]; };
int launch_lora_prep(alch_dtype dt, const LoraPrepParams& p, int n_jobs, hipStream_t stream);

// ---- attention ---------------------------------------------------------------------------
struct AttnArgs {
    alch_dtype dtype;
    int T, n_seqs, max_seqlen, Hq, Hkv, D;
    const int* cu_seqlens;       // device
    const int* cu_seqlens_host;  // host
    // shared prefixes: prefix[s] = -1 or the index of the earlier sequence whose keys and values every token
    // of s also attends to (device / host copies, both null when no sequence has a prefix)
    const int* prefix = nullptr;
    const int* prefix_host = nullptr;
    const void *Q, *K, *V, *O, *dO;  // dense [T, heads*D]
    const float* LSE;                // [T, Hq]
    float* delta;                    // scratch [2, T, Hq]: row sums of dO*O, produced inside launch_attn_bwd; the
                                     // matrix-core kernels keep LSE * log2(e) in the second half
    void *dQ, *dK, *dV;              // row stride ld_dqkv elements; dQ, dK, dV adjacent: [dQ | dK | dV] rows
    long long ld_dqkv;
    // rope_base > 0: dQ and dK come out already rotated by minus the RoPE angle (RoPE backward)
    const int* positions = nullptr;  // device [T] or null (index inside the sequence)
    float rope_base = 0.f;
};
int launch_attn_bwd(const AttnArgs& a, hipStream_t stream);
int launch_attn_bwd_generic(const AttnArgs& a, hipStream_t stream);
bool attn_mfma_supported(const AttnArgs& a);
int launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t stream);
static constexpr int kMaxPrefixSeqs = 4096;  // sequences per batch when prefixes are shared
double attn_pairs(int n_seqs, const int* cu_host, const int* prefix_host);
// forward: writes O [T,Hq*D] and LSE [T,Hq] for the query rows of sequences seq_begin .. n_seqs-1 (keys and
// values of a prefix sequence are read wherever it lies); prefix / prefix_host as in AttnArgs
int launch_attn_fwd_generic(alch_dtype dt, const void* Q, const void* K, const void* V, void* O, float* LSE, int T,
                            int n_seqs, const int* cu_seqlens, const int* cu_seqlens_host, const int* prefix,
                            int seq_begin, int Hq, int Hkv, int D, hipStream_t stream);
int launch_attn_fwd(alch_dtype dt, const void* Q, const void* K, const void* V, void* O, float* LSE, int T,
                    int n_seqs, int max_seqlen, const int* cu_seqlens, const int* cu_seqlens_host, const int* prefix,
                    const int* prefix_host, int seq_begin, int Hq, int Hkv, int D, hipStream_t stream);

// ---- LM head + cross-entropy ---------------------------------------------------------------
// n_counted[0] = #{t : labels[t] >= 0 and (mask == NULL or mask[t] != 0)}; row_loss[0..T) = 0
int launch_count_labels(const int* labels, const uint8_t* loss_mask, int T, int vocab, int* n_counted, float* row_loss,
                        hipStream_t stream);
// One chunk of logits rows [rows, vocab] (row stride ld), in place: logits -> dlogits =
// (softmax - onehot(label)) / N for counted rows, 0 otherwise; row_loss[r] = -log softmax[label].
int launch_ce_chunk(alch_dtype dt, void* logits, long long ld, int rows, int vocab, const int* labels,
                    const uint8_t* loss_mask, const int* n_counted, float* row_loss, hipStream_t stream,
                    const int* rows_dev = nullptr);
// counted[t] = label >= 0 and loss-mask byte nonzero; chunk_rows[c] = rows of chunk c among the first *n_rows rows
int launch_counted_mask(const int* labels, const uint8_t* loss_mask, int T, int vocab, uint8_t* counted, hipStream_t stream);
int launch_chunk_rows(const int* n_rows, int n_chunks, int chunk, int* chunk_rows, hipStream_t stream);
// dst[r] = src[index[r]] for r < min(*n_rows, T)
int launch_gather_int(const int* src, const int* index, const int* n_rows, int* dst, int T, hipStream_t stream);
// ---- DPO head on scored tokens (items) -----------------------------------------------------
// logp[m], logz[m] of a chunk of item logits rows
int launch_dpo_logp(alch_dtype dt, const void* logits, long long ld, int rows, int vocab, const int* labels, float* logp,
                    float* logz, hipStream_t stream);
// pi[slot] = sum of logp; z, loss, weight of every slot (w_slot [2 n_pairs]); z_out may be null
int launch_dpo_weights(const float* logp, const int* slots, const int* labels, int n_items, int vocab, const float* ref,
                       int n_pairs, float beta, float* pi, float* w_slot, float* z_out, float* loss_out, hipStream_t stream);
// a chunk of item logits rows -> their gradient, in place
int launch_dpo_grad(alch_dtype dt, void* logits, long long ld, int rows, int vocab, const int* labels, const int* slots,
                    const float* logz, const float* w_slot, int n_slots, hipStream_t stream);
// out [T, width] = 0, then out[item_row[m]] += src[m] (items sorted by row; fixed order)
int launch_dpo_scatter(alch_dtype dt, const void* src, const int* item_row, int n_items, void* out, int T, int width,
                       hipStream_t stream);

// loss_out[0] = sum(row_loss) / max(N, 1)   (fixed summation order)
int launch_finish_loss(const float* row_loss, const int* n_counted, float* loss_out, int T, hipStream_t stream);

}  // namespace alch
