// Low-rank adapter (LoRA) kernels: the rank-r products around a projection y = x W^T + s (x A^T) B^T
// (Section 3, assumption A1 and Section 6 of the paper: parameter-efficient fine-tuning, rank 8).
//
// With r = 8 every one of these products streams a [T, width] activation once and does 8 multiply-adds
// per element, so they are HBM-bound vector-ALU kernels, not matrix-core work:
//   down:  Y[T, r]  = alpha * X[T, K] * S         (S = A^T or B; "t1 = x A^T", "t2 = dy B")
//   up:    C[r, N]  = alpha * S[T, r]^T * X[T, N] (adapter gradients dA = t2^T x, dB^T = t1^T dy)
// Storage type T is float or bf16, arithmetic fp32, sums over tokens in a fixed order (deterministic).
#include "kernels.h"

namespace alch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_l;
typedef __attribute__((ext_vector_type(4))) float f32x4_l;

__device__ __forceinline__ void load8(const __bf16* p, float (&v)[8]) {
    const bf16x8_l t = *reinterpret_cast<const bf16x8_l*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)t[e];
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const f32x4_l a = *reinterpret_cast<const f32x4_l*>(p), b = *reinterpret_cast<const f32x4_l*>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}

// ---- down: 16 rows per work-group (4 per wavefront), 8 output columns per blockIdx.y ----------------
// S_KMAJOR: S(k, j) = S[j*lds + k] (the [r, K] matrix A), else S(k, j) = S[k*lds + j] (the [K, r] matrix B).
// Columns j >= r of the slot_cols-wide output slot are written as zeros (the slot is later read as a
// zero-padded operand of a matrix-core product).
template <typename T, bool S_KMAJOR>
__global__ __launch_bounds__(256) void k_lora_down(const T* __restrict__ X, long long ldx, int Trows, int K,
                                                   const T* __restrict__ S, long long lds, int r, float alpha,
                                                   T* __restrict__ Y, long long ldy) {
    __shared__ float red[4][64][33];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = blockIdx.y * 8;
    const long long t0 = (long long)blockIdx.x * 16 + wave * 4;
    if (j0 >= r) {
        if (lane < 32 && t0 + (lane >> 3) < Trows) Y[(t0 + (lane >> 3)) * ldy + j0 + (lane & 7)] = (T)0.f;
        return;
    }
    float acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int k0 = lane * 8; k0 < K; k0 += 512) {
        float x[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (t0 + i < Trows) {
                load8(X + (t0 + i) * ldx + k0, x[i]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[i][e] = 0.f;
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float s[8];
            if (S_KMAJOR) {  // q = output column: s = S(k0..k0+7, j0+q)
                load8(S + (long long)(j0 + q) * lds + k0, s);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][q] = __builtin_fmaf(x[i][e], s[e], acc[i][q]);
            } else {  // q = k index inside the chunk: s = S(k0+q, j0..j0+7)
                load8(S + (long long)(k0 + q) * lds + j0, s);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_fmaf(x[i][q], s[j], acc[i][j]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) red[wave][lane][i * 8 + j] = acc[i][j];
    __syncthreads();
    if (lane < 32) {
        float s = 0.f;
        for (int l = 0; l < 64; ++l) s += red[wave][l][lane];
        const long long t = t0 + (lane >> 3);
        if (t < Trows) Y[t * ldy + j0 + (lane & 7)] = (T)(alpha * s);
    }
}

// ---- up, pass 1: partial[jc][split][j][n] = sum over the rows of the split of S[t, 8*jc + j] * X[t, n] ----
// work-group = 512 columns (8 per lane) x one row split; its four wavefronts interleave the rows and
// fold their sums through LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void k_lora_up_partial(const T* __restrict__ S, long long lds, const T* __restrict__ X,
                                                         long long ldx, int Trows, int N, int rows_per_split,
                                                         float* __restrict__ partial) {
    __shared__ float red[3][64][65];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = blockIdx.x * 512 + lane * 8;
    const int split = blockIdx.y, nsplit = gridDim.y, jc = blockIdx.z;
    const long long r0 = (long long)split * rows_per_split;
    const long long r1 = r0 + rows_per_split < Trows ? r0 + rows_per_split : Trows;
    float acc[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[j][c] = 0.f;
    if (n0 < N) {
#pragma unroll 2
        for (long long t = r0 + wave; t < r1; t += 4) {
            float x[8], s[8];
            load8(X + t * ldx + n0, x);
            load8(S + t * lds + jc * 8, s);
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[j][c] = __builtin_fmaf(s[j], x[c], acc[j][c]);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int c = 0; c < 8; ++c) red[wave - 1][lane][j * 8 + c] = acc[j][c];
    }
    __syncthreads();
    if (wave == 0 && n0 < N) {
        float* out = partial + ((long long)(jc * nsplit + split) * 8) * N + n0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            f32x4_l lo, hi;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float v = ((acc[j][c] + red[0][lane][j * 8 + c]) + red[1][lane][j * 8 + c]) + red[2][lane][j * 8 + c];
                if (c < 4) lo[c] = v; else hi[c - 4] = v;
            }
            *reinterpret_cast<f32x4_l*>(out + (long long)j * N) = lo;
            *reinterpret_cast<f32x4_l*>(out + (long long)j * N + 4) = hi;
        }
    }
}

// ---- up, pass 2: C(j, n) (+)= alpha * sum over splits, written as C[j*ldc + n] or transposed C[n*ldc + j] ----
template <typename T>
__global__ __launch_bounds__(256) void k_lora_up_finish(const float* __restrict__ partial, int nsplit, int N, int r,
                                                        float alpha, T* __restrict__ C, long long ldc, int transposed,
                                                        int accumulate) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)N * r) return;
    // consecutive threads walk the contiguous index of the output
    const int jj = transposed ? (int)(idx % r) : (int)(idx / N);
    const int n = transposed ? (int)(idx / r) : (int)(idx % N);
    const float* p = partial + ((long long)(jj >> 3) * nsplit * 8 + (jj & 7)) * N + n;
    float s = 0.f;
    for (int k = 0; k < nsplit; ++k) s += p[(long long)k * 8 * N];
    T* dst = transposed ? C + (long long)n * ldc + jj : C + (long long)jj * ldc + n;
    s *= alpha;
    if (accumulate) s += (float)*dst;
    *dst = (T)s;
}

// ---- zero-padded stacked copy: dst[i, :] = i < r ? A[i, :] : 0 for i < rows_out (A may be null: all zeros) ----
template <typename T>
__global__ __launch_bounds__(256) void k_lora_pad_rows(const T* __restrict__ A, int r, int width, T* __restrict__ dst,
                                                       int rows_out) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)rows_out * width) return;
    const int i = (int)(idx / width);
    dst[idx] = (A && i < r) ? A[idx] : (T)0.f;
}

static int up_splits(int Trows, int N) {
    const int slabs = ceil_div(N, 512);
    int n = ceil_div(512, slabs);
    if (n < 4) n = 4;
    if (n > kLoraMaxSplits) n = kLoraMaxSplits;
    if (n > Trows) n = Trows > 0 ? Trows : 1;
    return n;
}

size_t lora_up_scratch_bytes(int rank, int n_max) {
    return (size_t)ceil_div(rank, 8) * kLoraMaxSplits * 8 * (size_t)n_max * sizeof(float);
}

template <typename T>
static int lora_down_t(const void* X, long long ldx, int Trows, int K, const void* S, long long lds, bool s_kmajor, int r,
                       float alpha, void* Y, long long ldy, int slot_cols, hipStream_t stream) {
    if (Trows <= 0) return ALCH_OK;
    const dim3 grid(ceil_div(Trows, 16), slot_cols / 8);
    if (s_kmajor)
        k_lora_down<T, true><<<grid, 256, 0, stream>>>((const T*)X, ldx, Trows, K, (const T*)S, lds, r, alpha, (T*)Y, ldy);
    else
        k_lora_down<T, false><<<grid, 256, 0, stream>>>((const T*)X, ldx, Trows, K, (const T*)S, lds, r, alpha, (T*)Y, ldy);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_lora_down(alch_dtype dt, const void* X, long long ldx, int Trows, int K, const void* S, long long lds,
                     bool s_kmajor, int r, float alpha, void* Y, long long ldy, int slot_cols, hipStream_t stream) {
    if (K % 8 || ldx % 8 || r % 8 || slot_cols % 8 || (S && lds % 8) || ldy % 8)
        return fail(ALCH_ERR_UNSUPPORTED, "adapter product: widths, strides and rank must be multiples of 8");
    return dt == ALCH_BF16 ? lora_down_t<__bf16>(X, ldx, Trows, K, S, lds, s_kmajor, r, alpha, Y, ldy, slot_cols, stream)
                           : lora_down_t<float>(X, ldx, Trows, K, S, lds, s_kmajor, r, alpha, Y, ldy, slot_cols, stream);
}

template <typename T>
static int lora_up_t(const void* S, long long lds, const void* X, long long ldx, int Trows, int N, int r, float alpha,
                     void* C, long long ldc, bool transposed, int accumulate, float* scratch, hipStream_t stream) {
    const int nsplit = Trows > 0 ? up_splits(Trows, N) : 0;
    if (nsplit > 0) {
        const int rps = ceil_div(Trows, nsplit);
        k_lora_up_partial<T><<<dim3(ceil_div(N, 512), nsplit, r / 8), 256, 0, stream>>>((const T*)S, lds, (const T*)X, ldx,
                                                                                       Trows, N, rps, scratch);
    }
    k_lora_up_finish<T><<<ceil_div((long long)N * r, 256LL), 256, 0, stream>>>(scratch, nsplit, N, r, alpha, (T*)C, ldc,
                                                                              transposed ? 1 : 0, accumulate);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_lora_up(alch_dtype dt, const void* S, long long lds, const void* X, long long ldx, int Trows, int N, int r,
                   float alpha, void* C, long long ldc, bool transposed, int accumulate, float* scratch,
                   hipStream_t stream) {
    if (N % 8 || ldx % 8 || lds % 8 || r % 8 || r <= 0)
        return fail(ALCH_ERR_UNSUPPORTED, "adapter gradient: widths, strides and rank must be multiples of 8");
    return dt == ALCH_BF16 ? lora_up_t<__bf16>(S, lds, X, ldx, Trows, N, r, alpha, C, ldc, transposed, accumulate, scratch, stream)
                           : lora_up_t<float>(S, lds, X, ldx, Trows, N, r, alpha, C, ldc, transposed, accumulate, scratch, stream);
}

int launch_lora_pad_rows(alch_dtype dt, const void* A, int r, int width, void* dst, int rows_out, hipStream_t stream) {
    const long long n = (long long)rows_out * width;
    if (n <= 0) return ALCH_OK;
    if (dt == ALCH_BF16)
        k_lora_pad_rows<__bf16><<<ceil_div(n, 256LL), 256, 0, stream>>>((const __bf16*)A, r, width, (__bf16*)dst, rows_out);
    else
        k_lora_pad_rows<float><<<ceil_div(n, 256LL), 256, 0, stream>>>((const float*)A, r, width, (float*)dst, rows_out);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
