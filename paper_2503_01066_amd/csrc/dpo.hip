// DPO head on scored tokens (Section 6 of the paper: DPO is the example loss of preference alignment;
// Section 4.1: the loss is computed on the response tokens, which sit on the saved prefill of their prompt).
//
// A scored token is an item (row, label, slot): the log-probability of `label` under the LM-head row computed
// from stack-output row `row` adds to pi[slot]; slots 2p and 2p+1 are the chosen and the rejected response of
// pair p.  With z_p = beta [(pi_2p - ref_2p) - (pi_2p+1 - ref_2p+1)] the loss is mean_p -log sigmoid(z_p), and
// the gradient with respect to an item's logits is w (onehot(label) - softmax) with
// w = -/+ beta sigmoid(-z_p) / n_pairs for the chosen / rejected slot.  An item with a label or slot out of
// range scores nothing.  All sums run in a fixed order: results are deterministic.
#include "kernels.h"

namespace alch {

template <typename T> __device__ __forceinline__ float ldf(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v) { *p = (T)v; }

// block-wide reductions of 256 threads, every thread gets the result
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// logz[m] = log sum_v exp(logits[m, v]);  logp[m] = logits[m, label] - logz[m]  (0 for a label out of range)
template <typename T>
__global__ __launch_bounds__(256) void k_dpo_logp(const T* __restrict__ logits, long long ld, int vocab,
                                                  const int* __restrict__ labels, float* __restrict__ logp,
                                                  float* __restrict__ logz) {
    __shared__ float red[4];
    const int m = blockIdx.x;
    const T* row = logits + (long long)m * ld;
    float mx = -INFINITY;
    for (int v = threadIdx.x; v < vocab; v += 256) mx = fmaxf(mx, ldf(row + v));
    mx = block_max(mx, red);
    float s = 0.f;
    for (int v = threadIdx.x; v < vocab; v += 256) s += __expf(ldf(row + v) - mx);
    s = block_sum(s, red);
    if (threadIdx.x == 0) {
        const float lz = mx + __logf(s);
        const int label = labels[m];
        logz[m] = lz;
        logp[m] = (label >= 0 && label < vocab) ? ldf(row + label) - lz : 0.f;
    }
}

// pi[slot] = sum of logp over the items of that slot (one work-group per slot)
__global__ __launch_bounds__(256) void k_dpo_slot_sums(const float* __restrict__ logp, const int* __restrict__ slots,
                                                       const int* __restrict__ labels, int n_items, int vocab,
                                                       float* __restrict__ pi) {
    __shared__ float red[4];
    const int slot = blockIdx.x;
    float s = 0.f;
    for (int m = threadIdx.x; m < n_items; m += 256)
        if (slots[m] == slot && labels[m] >= 0 && labels[m] < vocab) s += logp[m];
    s = block_sum(s, red);
    if (threadIdx.x == 0) pi[slot] = s;
}

// z, the loss and the weight of every slot (single work-group)
__global__ __launch_bounds__(256) void k_dpo_finish(const float* __restrict__ pi, const float* __restrict__ ref, int n_pairs,
                                                    float beta, float* __restrict__ w_slot, float* __restrict__ z_out,
                                                    float* __restrict__ loss_out) {
    __shared__ float red[4];
    float part = 0.f;
    for (int p = threadIdx.x; p < n_pairs; p += 256) {
        const float z = beta * ((pi[2 * p] - ref[2 * p]) - (pi[2 * p + 1] - ref[2 * p + 1]));
        part += fmaxf(-z, 0.f) + log1pf(__expf(-fabsf(z)));      // -log sigmoid(z)
        const float dz = -1.f / (1.f + __expf(z)) / (float)n_pairs;  // d loss / d z
        w_slot[2 * p] = beta * dz;
        w_slot[2 * p + 1] = -beta * dz;
        if (z_out) z_out[p] = z;
    }
    part = block_sum(part, red);
    if (threadIdx.x == 0) loss_out[0] = n_pairs > 0 ? part / (float)n_pairs : 0.f;
}

// logits row -> its gradient, in place: w (onehot(label) - softmax)
template <typename T>
__global__ __launch_bounds__(256) void k_dpo_grad(T* __restrict__ logits, long long ld, int vocab,
                                                  const int* __restrict__ labels, const int* __restrict__ slots,
                                                  const float* __restrict__ logz, const float* __restrict__ w_slot,
                                                  int n_slots) {
    const int m = blockIdx.x;
    T* row = logits + (long long)m * ld;
    const int label = labels[m], slot = slots[m];
    const bool scored = label >= 0 && label < vocab && slot >= 0 && slot < n_slots;
    const float w = scored ? w_slot[slot] : 0.f;
    const float lz = logz[m];
    for (int v = threadIdx.x; v < vocab; v += 256) {
        float g = -w * __expf(ldf(row + v) - lz);
        if (v == label) g += w;
        stf(row + v, g);
    }
}

// bf16 fast paths of the two kernels above: one 1024-thread work-group per row, 16-byte accesses.  The
// log-probability kernel keeps the row in registers (up to 16 chunks of 8 logits per thread, vocab <= 131072),
// so it reads the logits once; the gradient kernel streams them.  Both need vocab and ld to be multiples of 8
// and a 16-byte aligned base.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_d;
static constexpr int kRowThreads = 1024, kRowChunks = 16;

__global__ __launch_bounds__(kRowThreads) void k_dpo_logp_bf16_row(const __bf16* __restrict__ logits, long long ld, int vocab,
                                                                    const int* __restrict__ labels, float* __restrict__ logp,
                                                                    float* __restrict__ logz) {
    __shared__ float red[kRowThreads / 64];
    const int m = blockIdx.x;
    const __bf16* row = logits + (long long)m * ld;
    const int nchunks = vocab >> 3;
    bf16x8_d x[kRowChunks];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < kRowChunks; ++k) {
        const int c = threadIdx.x + k * kRowThreads;
        if (c < nchunks) {
            x[k] = *reinterpret_cast<const bf16x8_d*>(row + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) mx = fmaxf(mx, (float)x[k][e]);
        }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = red[0];
#pragma unroll
    for (int w = 1; w < kRowThreads / 64; ++w) mx = fmaxf(mx, red[w]);
    __syncthreads();
    // (the empty asm keeps the row packed in registers: without it the compiler carries fp32 copies across)
#pragma unroll
    for (int k = 0; k < kRowChunks; ++k) asm volatile("" : "+v"(x[k]));
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kRowChunks; ++k) {
        const int c = threadIdx.x + k * kRowThreads;
        if (c < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s += __expf((float)x[k][e] - mx);
        }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        s = 0.f;
        for (int w = 0; w < kRowThreads / 64; ++w) s += red[w];
        const float lz = mx + __logf(s);
        const int label = labels[m];
        logz[m] = lz;
        logp[m] = (label >= 0 && label < vocab) ? (float)row[label] - lz : 0.f;
    }
}

__global__ __launch_bounds__(kRowThreads) void k_dpo_grad_bf16_row(__bf16* __restrict__ logits, long long ld, int vocab,
                                                                    const int* __restrict__ labels, const int* __restrict__ slots,
                                                                    const float* __restrict__ logz, const float* __restrict__ w_slot,
                                                                    int n_slots) {
    const int m = blockIdx.x;
    __bf16* row = logits + (long long)m * ld;
    const int label = labels[m], slot = slots[m];
    const bool scored = label >= 0 && label < vocab && slot >= 0 && slot < n_slots;
    const float w = scored ? w_slot[slot] : 0.f;
    const float lz = logz[m];
    const int nchunks = vocab >> 3;
    for (int c = threadIdx.x; c < nchunks; c += kRowThreads) {
        bf16x8_d x = *reinterpret_cast<const bf16x8_d*>(row + c * 8), g;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = -w * __expf((float)x[e] - lz);
            if (c * 8 + e == label) v += w;
            g[e] = (__bf16)v;
        }
        *reinterpret_cast<bf16x8_d*>(row + c * 8) = g;
    }
}

static bool rows_vectorisable(const void* logits, long long ld, int vocab) {
    return vocab % 8 == 0 && ld % 8 == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;
}

// out[row, :] = sum of src[m, :] over the run of items with item_row[m] == row (items sorted by row); the
// first item of a run does the sum.  Rows without an item keep the zeros written before.
template <typename T>
__global__ __launch_bounds__(256) void k_dpo_scatter(const T* __restrict__ src, const int* __restrict__ item_row, int n_items,
                                                     T* __restrict__ out, int width) {
    const int m = blockIdx.x;
    const int row = item_row[m];
    if (m > 0 && item_row[m - 1] == row) return;
    int end = m + 1;
    while (end < n_items && item_row[end] == row) ++end;
    for (int c = threadIdx.x; c < width; c += 256) {
        float s = 0.f;
        for (int k = m; k < end; ++k) s += ldf(src + (long long)k * width + c);
        stf(out + (long long)row * width + c, s);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_fill_zero(T* __restrict__ x, long long n) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) x[i] = (T)0.f;
}

int launch_dpo_logp(alch_dtype dt, const void* logits, long long ld, int rows, int vocab, const int* labels, float* logp,
                    float* logz, hipStream_t stream) {
    if (rows <= 0) return ALCH_OK;
    if (dt == ALCH_BF16 && rows_vectorisable(logits, ld, vocab) && vocab <= 8 * kRowThreads * kRowChunks)
        k_dpo_logp_bf16_row<<<rows, kRowThreads, 0, stream>>>((const __bf16*)logits, ld, vocab, labels, logp, logz);
    else if (dt == ALCH_BF16) k_dpo_logp<__bf16><<<rows, 256, 0, stream>>>((const __bf16*)logits, ld, vocab, labels, logp, logz);
    else k_dpo_logp<float><<<rows, 256, 0, stream>>>((const float*)logits, ld, vocab, labels, logp, logz);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_dpo_weights(const float* logp, const int* slots, const int* labels, int n_items, int vocab, const float* ref,
                       int n_pairs, float beta, float* pi, float* w_slot, float* z_out, float* loss_out, hipStream_t stream) {
    if (n_pairs > 0) k_dpo_slot_sums<<<2 * n_pairs, 256, 0, stream>>>(logp, slots, labels, n_items, vocab, pi);
    k_dpo_finish<<<1, 256, 0, stream>>>(pi, ref, n_pairs, beta, w_slot, z_out, loss_out);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_dpo_grad(alch_dtype dt, void* logits, long long ld, int rows, int vocab, const int* labels, const int* slots,
                    const float* logz, const float* w_slot, int n_slots, hipStream_t stream) {
    if (rows <= 0) return ALCH_OK;
    if (dt == ALCH_BF16 && rows_vectorisable(logits, ld, vocab))
        k_dpo_grad_bf16_row<<<rows, kRowThreads, 0, stream>>>((__bf16*)logits, ld, vocab, labels, slots, logz, w_slot, n_slots);
    else if (dt == ALCH_BF16) k_dpo_grad<__bf16><<<rows, 256, 0, stream>>>((__bf16*)logits, ld, vocab, labels, slots, logz, w_slot, n_slots);
    else k_dpo_grad<float><<<rows, 256, 0, stream>>>((float*)logits, ld, vocab, labels, slots, logz, w_slot, n_slots);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_dpo_scatter(alch_dtype dt, const void* src, const int* item_row, int n_items, void* out, int T, int width,
                       hipStream_t stream) {
    const long long n = (long long)T * width;
    if (n <= 0) return ALCH_OK;
    const int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    if (dt == ALCH_BF16) {
        k_fill_zero<__bf16><<<grid, 256, 0, stream>>>((__bf16*)out, n);
        if (n_items > 0) k_dpo_scatter<__bf16><<<n_items, 256, 0, stream>>>((const __bf16*)src, item_row, n_items, (__bf16*)out, width);
    } else {
        k_fill_zero<float><<<grid, 256, 0, stream>>>((float*)out, n);
        if (n_items > 0) k_dpo_scatter<float><<<n_items, 256, 0, stream>>>((const float*)src, item_row, n_items, (float*)out, width);
    }
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
