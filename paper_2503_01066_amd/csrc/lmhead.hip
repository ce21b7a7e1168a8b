// Cross-entropy on chunks of LM-head logits (Section 5 of the paper: the continual-pre-training
// loss is computed from the saved prefill output and the prompt's own tokens as labels).
// Logits are produced chunk by chunk by the GEMM and turned into their gradient in place, so the
// [tokens, vocab] matrix is never stored whole.
#include "kernels.h"

namespace alch {

template <typename T> __device__ __forceinline__ float ldf(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v) { *p = (T)v; }

__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}
__device__ __forceinline__ float wsum2(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// A position counts when its label names a vocabulary entry (0 <= label < vocab) and its loss-mask byte, if a
// mask is given, is nonzero: one predicate for the count, the counted mask and the row kernels.
__device__ __forceinline__ bool label_counts(int label, int vocab) { return (unsigned)label < (unsigned)vocab; }

__global__ __launch_bounds__(256) void k_count_labels(const int* __restrict__ labels, const uint8_t* __restrict__ mask,
                                                      int T, int vocab, int* __restrict__ n_counted,
                                                      float* __restrict__ row_loss) {
    // single block: deterministic count
    __shared__ int part[4];
    int c = 0;
    for (int t = threadIdx.x; t < T; t += 256) {
        c += (label_counts(labels[t], vocab) && (!mask || mask[t] != 0)) ? 1 : 0;
        row_loss[t] = 0.f;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) c += __shfl_xor(c, d, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) n_counted[0] = part[0] + part[1] + part[2] + part[3];
}

template <typename T>
__global__ __launch_bounds__(256) void k_ce_chunk(T* __restrict__ logits, long long ld, int vocab,
                                                  const int* __restrict__ labels, const uint8_t* __restrict__ mask,
                                                  const int* __restrict__ n_counted, float* __restrict__ row_loss,
                                                  const int* __restrict__ rows_dev) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    if (rows_dev && r >= *rows_dev) return;  // row count decided on the device (compacted rows)
    T* row = logits + (long long)r * ld;
    const int label = labels[r];
    const bool counted = label_counts(label, vocab) && (!mask || mask[r] != 0);
    if (!counted) {
        for (int v = threadIdx.x; v < vocab; v += 256) row[v] = (T)0.f;
        return;
    }
    float m = -INFINITY;
    for (int v = threadIdx.x; v < vocab; v += 256) m = fmaxf(m, ldf(row + v));
    m = wmax(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int v = threadIdx.x; v < vocab; v += 256) s += __expf(ldf(row + v) - m);
    s = wsum2(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    s = red[0] + red[1] + red[2] + red[3];
    const float logz = m + __logf(s);
    const float inv_n = 1.f / (float)n_counted[0];
    const float x_label = ldf(row + label);
    __syncthreads();  // everyone has read the label logit before it is overwritten
    for (int v = threadIdx.x; v < vocab; v += 256) {
        float p = __expf(ldf(row + v) - logz);
        if (v == label) p -= 1.f;
        stf(row + v, p * inv_n);
    }
    if (threadIdx.x == 0) row_loss[r] = logz - x_label;
}

// bf16 fast path: one 1024-thread work-group per row keeps the whole row in registers (up to 16 chunks of
// 8 logits per thread, i.e. vocab <= 131072), so the logits are read once and the gradient written once:
// the three passes (max, sum of exponentials, gradient) run on registers.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_c;
static constexpr int kCeThreads = 1024, kCeChunks = 16;
__global__ __launch_bounds__(kCeThreads) void k_ce_chunk_bf16_row(__bf16* __restrict__ logits, long long ld, int vocab,
                                                                   const int* __restrict__ labels,
                                                                   const uint8_t* __restrict__ mask,
                                                                   const int* __restrict__ n_counted,
                                                                   float* __restrict__ row_loss,
                                                                   const int* __restrict__ rows_dev) {
    __shared__ float red[kCeThreads / 64];
    const int r = blockIdx.x;
    if (rows_dev && r >= *rows_dev) return;  // row count decided on the device (compacted rows)
    __bf16* row = logits + (long long)r * ld;
    const int label = labels[r];
    const bool counted = label_counts(label, vocab) && (!mask || mask[r] != 0);
    const int nchunks = vocab >> 3;
    if (!counted) {
        bf16x8_c z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
        for (int c = threadIdx.x; c < nchunks; c += kCeThreads) *reinterpret_cast<bf16x8_c*>(row + c * 8) = z;
        return;
    }
    bf16x8_c x[kCeChunks];
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < kCeChunks; ++k) {
        const int c = threadIdx.x + k * kCeThreads;
        if (c < nchunks) {
            x[k] = *reinterpret_cast<const bf16x8_c*>(row + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) m = fmaxf(m, (float)x[k][e]);
        }
    }
    m = wmax(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int w = 1; w < kCeThreads / 64; ++w) m = fmaxf(m, red[w]);
    __syncthreads();
    const float kL2e = 1.4426950408889634f;
    float s = 0.f;
    // (the empty asm keeps the row packed in registers between passes: without it the compiler carries the
    // converted fp32 copies across and runs out of registers)
#pragma unroll
    for (int k = 0; k < kCeChunks; ++k) asm volatile("" : "+v"(x[k]));
#pragma unroll
    for (int k = 0; k < kCeChunks; ++k) {
        const int c = threadIdx.x + k * kCeThreads;
        if (c < nchunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s += __builtin_amdgcn_exp2f(((float)x[k][e] - m) * kL2e);
        }
    }
    s = wsum2(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    s = 0.f;
#pragma unroll
    for (int w = 0; w < kCeThreads / 64; ++w) s += red[w];
    const float logz = m + __logf(s);
    const float inv_n = 1.f / (float)n_counted[0];
#pragma unroll
    for (int k = 0; k < kCeChunks; ++k) asm volatile("" : "+v"(x[k]));
#pragma unroll
    for (int k = 0; k < kCeChunks; ++k) {
        const int c = threadIdx.x + k * kCeThreads;
        if (c < nchunks) {
            bf16x8_c o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float pr = __builtin_amdgcn_exp2f(((float)x[k][e] - logz) * kL2e);
                if (c * 8 + e == label) {
                    pr -= 1.f;
                    row_loss[r] = logz - (float)x[k][e];
                }
                o[e] = (__bf16)(pr * inv_n);
            }
            *reinterpret_cast<bf16x8_c*>(row + c * 8) = o;
        }
    }
}

__global__ __launch_bounds__(256) void k_finish_loss(const float* __restrict__ row_loss, const int* __restrict__ n_counted,
                                                     float* __restrict__ loss_out, int T) {
    __shared__ float red[4];
    float s = 0.f;
    for (int t = threadIdx.x; t < T; t += 256) s += row_loss[t];
    s = wsum2(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int n = n_counted[0];
        loss_out[0] = n > 0 ? (red[0] + red[1] + red[2] + red[3]) / (float)n : 0.f;
    }
}

// counted[t] = 1 where the token contributes to the loss (0 <= label < vocab and loss-mask byte nonzero)
__global__ __launch_bounds__(256) void k_counted_mask(const int* __restrict__ labels, const uint8_t* __restrict__ mask,
                                                      int T, int vocab, uint8_t* __restrict__ counted) {
    for (int t = blockIdx.x * 256 + threadIdx.x; t < T; t += gridDim.x * 256)
        counted[t] = (label_counts(labels[t], vocab) && (!mask || mask[t] != 0)) ? 1 : 0;
}
// chunk_rows[c] = number of the n compacted rows that fall into row chunk c
__global__ void k_chunk_rows(const int* __restrict__ n_rows, int n_chunks, int chunk, int* __restrict__ chunk_rows) {
    const int n = n_rows[0];
    for (int c = threadIdx.x; c < n_chunks; c += blockDim.x) {
        const int left = n - c * chunk;
        chunk_rows[c] = left < 0 ? 0 : (left > chunk ? chunk : left);
    }
}
// dst[r] = src[index[r]] for r < *n_rows
__global__ __launch_bounds__(256) void k_gather_int(const int* __restrict__ src, const int* __restrict__ index,
                                                    const int* __restrict__ n_rows, int* __restrict__ dst, int T) {
    const int n = min(n_rows[0], T);
    for (int r = blockIdx.x * 256 + threadIdx.x; r < n; r += gridDim.x * 256) dst[r] = src[index[r]];
}
int launch_gather_int(const int* src, const int* index, const int* n_rows, int* dst, int T, hipStream_t stream) {
    if (T <= 0) return ALCH_OK;
    k_gather_int<<<ceil_div(T, 256) < 1024 ? ceil_div(T, 256) : 1024, 256, 0, stream>>>(src, index, n_rows, dst, T);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}
int launch_counted_mask(const int* labels, const uint8_t* loss_mask, int T, int vocab, uint8_t* counted, hipStream_t stream) {
    if (T <= 0) return ALCH_OK;
    k_counted_mask<<<ceil_div(T, 256) < 1024 ? ceil_div(T, 256) : 1024, 256, 0, stream>>>(labels, loss_mask, T, vocab, counted);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}
int launch_chunk_rows(const int* n_rows, int n_chunks, int chunk, int* chunk_rows, hipStream_t stream) {
    if (n_chunks <= 0) return ALCH_OK;
    k_chunk_rows<<<1, 64, 0, stream>>>(n_rows, n_chunks, chunk, chunk_rows);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_count_labels(const int* labels, const uint8_t* loss_mask, int T, int vocab, int* n_counted, float* row_loss,
                        hipStream_t stream) {
    k_count_labels<<<1, 256, 0, stream>>>(labels, loss_mask, T, vocab, n_counted, row_loss);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_ce_chunk(alch_dtype dt, void* logits, long long ld, int rows, int vocab, const int* labels,
                    const uint8_t* loss_mask, const int* n_counted, float* row_loss, hipStream_t stream,
                    const int* rows_dev) {
    if (rows <= 0) return ALCH_OK;
    if (dt == ALCH_BF16 && vocab % 8 == 0 && ld % 8 == 0 && vocab <= kCeThreads * kCeChunks * 8 && aligned16(logits))
        k_ce_chunk_bf16_row<<<rows, kCeThreads, 0, stream>>>((__bf16*)logits, ld, vocab, labels, loss_mask, n_counted, row_loss, rows_dev);
    else if (dt == ALCH_BF16)
        k_ce_chunk<__bf16><<<rows, 256, 0, stream>>>((__bf16*)logits, ld, vocab, labels, loss_mask, n_counted, row_loss, rows_dev);
    else
        k_ce_chunk<float><<<rows, 256, 0, stream>>>((float*)logits, ld, vocab, labels, loss_mask, n_counted, row_loss, rows_dev);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_finish_loss(const float* row_loss, const int* n_counted, float* loss_out, int T, hipStream_t stream) {
    k_finish_loss<<<1, 256, 0, stream>>>(row_loss, n_counted, loss_out, T);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
