// Low-rank adapter (LoRA) kernels: the rank-r products around a projection y = x W^T + s (x A^T) B^T
// (Section 3, assumption A1 and Section 6 of the paper: parameter-efficient fine-tuning, rank 8).
//
// With r = 8 every one of these products streams a [T, width] activation once and does 8 multiply-adds
// per element, so they are HBM-bound vector-ALU kernels, not matrix-core work:
//   down:  Y[T, r]  = alpha * X[T, K] * S         (S = A^T or B; "t1 = x A^T", "t2 = dy B")
//   up:    C[r, N]  = alpha * S[T, r]^T * X[T, N] (adapter gradients dA = t2^T x, dB^T = t1^T dy)
// Storage type T is float or bf16, arithmetic fp32, sums over tokens in a fixed order (deterministic).
#include <algorithm>

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

// ---- down, vector-ALU version (any dtype): 16 rows per work-group (4 per wavefront), 8 output columns
// per blockIdx.y.  S(k, j) = S[j*lds + k] (an [r, K] matrix: A, or B transposed).  Columns j >= r of the
// slot_cols-wide output slot are written as zeros (the slot is later read as a zero-padded operand of a
// matrix-core product).
template <typename T>
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
            load8(S + (long long)(j0 + q) * lds + k0, s);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][q] = __builtin_fmaf(x[i][e], s[e], acc[i][q]);
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

// ---- down on the matrix cores (bf16, K a multiple of 64): eight multiply-adds per streamed element are
// too many for the vector ALU to keep up with HBM, so the [32 rows x 16 k] x [16 k x 32 columns] MFMA does
// them (columns >= r are zero operands).  A work-group owns 32 rows; its four wavefronts split K and fold
// their sums through LDS in a fixed order.  Up to three (X, S, Y) problems per launch (blockIdx.z).
typedef __attribute__((ext_vector_type(16))) float f32x16_l;
struct LoraDownJob {
    const __bf16* X; long long ldx; int K;
    const __bf16* S; long long lds; int r;   // r = 0: zero-fill the slot
    __bf16* Y;
};
struct LoraDownParams {
    LoraDownJob job[3];
    int Trows; long long ldy; float alpha; int slot_cols;
};
__global__ __launch_bounds__(256) void k_lora_down_mfma(LoraDownParams p) {
    __shared__ float red[3][64][17];
    const LoraDownJob jb = p.job[blockIdx.z];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, kh = lane >> 5;
    const long long t0 = (long long)blockIdx.x * 32;
    const int j0 = blockIdx.y * 32;  // first output column of this pass
    f32x16_l acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    if (j0 < jb.r) {
        const int kq = jb.K / 4;  // this wave's share of K (a multiple of 16)
        // rows past the end and columns past r read a valid row instead: their results are never stored
        const long long tr = t0 + c < p.Trows ? t0 + c : p.Trows - 1;
        const int jc = j0 + c < jb.r ? j0 + c : 0;
        const __bf16* xp = jb.X + tr * jb.ldx + wave * kq + 8 * kh;
        const __bf16* sp = jb.S + (long long)jc * jb.lds + wave * kq + 8 * kh;
        // batches of 128 k (eight 16-byte loads of X and of S per lane), double buffered: the loads of
        // the next batch are in flight while the matrix instructions consume the current one
        auto load_batch = [&](bf16x8_l (&a)[8], bf16x8_l (&b)[8], int kb) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                a[u] = *reinterpret_cast<const bf16x8_l*>(xp + kb + 16 * u);
                b[u] = *reinterpret_cast<const bf16x8_l*>(sp + kb + 16 * u);
            }
        };
        auto mma_batch = [&](const bf16x8_l (&a)[8], const bf16x8_l (&b)[8]) {
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u], acc, 0, 0, 0);
        };
        const int nb = kq / 128;
        bf16x8_l a0[8], b0[8], a1[8], b1[8];
        if (nb > 0) load_batch(a0, b0, 0);
        int i = 0;
        for (; i + 2 <= nb; i += 2) {
            load_batch(a1, b1, (i + 1) * 128);
            __builtin_amdgcn_sched_barrier(0);
            mma_batch(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (i + 2 < nb) load_batch(a0, b0, (i + 2) * 128);
            __builtin_amdgcn_sched_barrier(0);
            mma_batch(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (i < nb) mma_batch(a0, b0);
        int k = nb * 128;
        for (; k < kq; k += 16) {
            const bf16x8_l a = *reinterpret_cast<const bf16x8_l*>(xp + k);
            const bf16x8_l b = *reinterpret_cast<const bf16x8_l*>(sp + k);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) red[wave - 1][lane][e] = acc[e];
    }
    __syncthreads();
    if (wave == 0) {
        // accumulator element e: row 8*(e>>2) + 4*kh + (e&3), column c
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float v = ((acc[e] + red[0][lane][e]) + red[1][lane][e]) + red[2][lane][e];
            const long long t = t0 + 8 * (e >> 2) + 4 * kh + (e & 3);
            if (t < p.Trows && j0 + c < p.slot_cols) jb.Y[t * p.ldy + j0 + c] = (__bf16)(j0 + c < jb.r ? p.alpha * v : 0.f);
        }
    }
}

// ---- up, pass 1: partial[jc][split][j][n] = sum over the rows of the split of S[t, 8*jc + j] * X[t, n] ----
// work-group = 512 columns (8 per lane) x one row split; its four wavefronts interleave the rows and
// fold their sums through LDS in a fixed order.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_l;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_l;

// One token (float storage) or one pair of tokens (bf16 storage) of the rank-8 outer-product sum
// acc[j][c] += S[t, j] * X[t, c].  For bf16 the two tokens of a pair are interleaved into (t, t+1)
// halfword pairs (one byte-permute per pair) and each 2-term sum is one packed dot-product instruction
// accumulating in fp32: half the vector instructions of convert + multiply-add per element.
__device__ __forceinline__ void up_step(const float* xr, const float* sr, long long, long long, bool, float (&acc)[8][8]) {
    float x[8], s[8];
    load8(xr, x);
    load8(sr, s);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[j][c] = __builtin_fmaf(s[j], x[c], acc[j][c]);
}
__device__ __forceinline__ void up_step(const __bf16* xr, const __bf16* sr, long long ldx, long long lds, bool second,
                                        float (&acc)[8][8]) {
    const u32x4_l zero = {0u, 0u, 0u, 0u};
    const u32x4_l x0 = *reinterpret_cast<const u32x4_l*>(xr), s0 = *reinterpret_cast<const u32x4_l*>(sr);
    const u32x4_l x1 = second ? *reinterpret_cast<const u32x4_l*>(xr + ldx) : zero;
    const u32x4_l s1 = second ? *reinterpret_cast<const u32x4_l*>(sr + lds) : zero;
    unsigned xp[8], sp[8];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        xp[2 * m] = __builtin_amdgcn_perm(x1[m], x0[m], 0x05040100u);      // (x[t][2m],   x[t+1][2m])
        xp[2 * m + 1] = __builtin_amdgcn_perm(x1[m], x0[m], 0x07060302u);  // (x[t][2m+1], x[t+1][2m+1])
        sp[2 * m] = __builtin_amdgcn_perm(s1[m], s0[m], 0x05040100u);
        sp[2 * m + 1] = __builtin_amdgcn_perm(s1[m], s0[m], 0x07060302u);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c)
            acc[j][c] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_l, sp[j]), __builtin_bit_cast(bf16x2_l, xp[c]),
                                                        acc[j][c], false);
}
template <typename T> struct UpStep { static constexpr int kTokens = 1; };
template <> struct UpStep<__bf16> { static constexpr int kTokens = 2; };

struct LoraUpJob {
    const void* S; long long lds;
    const void* X; long long ldx;
    int N, nsplit, rows_per_split;
    void* C; long long ldc;
    int transposed;
    long long scratch_off;  // floats
};
struct LoraUpParams {
    LoraUpJob job[kLoraUpJobs];
    int Trows, r, accumulate;
    float alpha;
    float* scratch;
};

// blockIdx.z = job * (r / 8) + chunk of eight rank rows; work-groups beyond a job's column slabs or row splits exit
template <typename T>
__global__ __launch_bounds__(256) void k_lora_up_partial(LoraUpParams p) {
    __shared__ float red[3][64][65];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunks = p.r >> 3;
    const LoraUpJob jb = p.job[blockIdx.z / chunks];
    const int jc = blockIdx.z % chunks;
    const int N = jb.N, nsplit = jb.nsplit, split = blockIdx.y;
    if ((int)blockIdx.x * 512 >= N || split >= nsplit) return;
    const T* __restrict__ S = static_cast<const T*>(jb.S);
    const T* __restrict__ X = static_cast<const T*>(jb.X);
    const long long lds = jb.lds, ldx = jb.ldx;
    const int Trows = p.Trows, rows_per_split = jb.rows_per_split;
    float* __restrict__ partial = p.scratch + jb.scratch_off;
    const int n0 = blockIdx.x * 512 + lane * 8;
    const long long r0 = (long long)split * rows_per_split;
    const long long r1 = r0 + rows_per_split < Trows ? r0 + rows_per_split : Trows;
    constexpr int kTok = UpStep<T>::kTokens;
    float acc[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[j][c] = 0.f;
    if (n0 < N) {
#pragma unroll 2
        for (long long t = r0 + wave * kTok; t < r1; t += 4 * kTok)
            up_step(X + t * ldx + n0, S + t * lds + jc * 8, ldx, lds, t + 1 < r1, acc);
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

// ---- up, pass 2: C(j, n) (+)= alpha * sum over splits, written as C[j*ldc + n] or transposed C[n*ldc + j].
// Eight lanes share one output: lane q adds splits q, q+8, ... and the eight sums are folded in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void k_lora_up_finish(LoraUpParams p) {
    const LoraUpJob jb = p.job[blockIdx.y];
    const int N = jb.N, nsplit = jb.nsplit, r = p.r, transposed = jb.transposed, accumulate = p.accumulate;
    const float alpha = p.alpha;
    const float* __restrict__ partial = p.scratch + jb.scratch_off;
    T* __restrict__ C = static_cast<T*>(jb.C);
    const long long ldc = jb.ldc;
    const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) >> 3;
    const int q = threadIdx.x & 7;
    const bool live = idx < (long long)N * r;
    // consecutive outputs walk n: the partial sums are read in order (C itself is small)
    const int jj = !live ? 0 : (int)(idx / N);
    const int n = !live ? 0 : (int)(idx % N);
    const float* src = partial + ((long long)(jj >> 3) * nsplit * 8 + (jj & 7)) * N + n;
    float s = 0.f;
    if (live)
        for (int k = q; k < nsplit; k += 8) s += src[(long long)k * 8 * N];
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    s += __shfl_xor(s, 4, 64);
    if (live && q == 0) {
        T* dst = transposed ? C + (long long)n * ldc + jj : C + (long long)jj * ldc + n;
        s *= alpha;
        if (accumulate) s += (float)*dst;
        *dst = (T)s;
    }
}

// ---- operand preparation, all adapters of a layer in one launch: job z writes dst [rows_out, cols] with
// dst[i, c] = i < r ? (transpose ? src[c*r + i] : src[i*cols + c]) : 0   (src null: all zeros).
// Used for the zero-padded stacks of the A matrices (extra operand of the data-gradient products) and for
// B^T (so that both rank-r "down" products read an [r, K] matrix).
template <typename T>
__global__ __launch_bounds__(256) void k_lora_prep(LoraPrepParams p) {
    const LoraPrepJob jb = p.job[blockIdx.y];
    const long long n = (long long)jb.rows_out * jb.cols;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (long long)gridDim.x * 256) {
        const int i = (int)(idx / jb.cols), c = (int)(idx % jb.cols);
        const T* src = static_cast<const T*>(jb.src);
        T v = (T)0.f;
        if (src && i < jb.r) v = jb.transpose ? src[(long long)c * jb.r + i] : src[idx];
        static_cast<T*>(jb.dst)[idx] = v;
    }
}

static int up_splits(int Trows, int N) {
    const int slabs = ceil_div(N, 512);
    int n = ceil_div(256, slabs);
    if (n < 4) n = 4;
    if (n > kLoraMaxSplits) n = kLoraMaxSplits;
    if (n > Trows) n = Trows > 0 ? Trows : 1;
    return n;
}

size_t lora_up_scratch_bytes(int rank, int n_sum) {
    return (size_t)ceil_div(rank, 8) * kLoraMaxSplits * 8 * (size_t)n_sum * sizeof(float);
}

template <typename T>
static int lora_down_valu(const LoraDown& j, int Trows, float alpha, long long ldy, int slot_cols, hipStream_t stream) {
    const dim3 grid(ceil_div(Trows, 16), slot_cols / 8);
    k_lora_down<T><<<grid, 256, 0, stream>>>((const T*)j.X, j.ldx, Trows, j.K, (const T*)j.S, j.lds, j.r, alpha, (T*)j.Y, ldy);
    return ALCH_OK;
}

int launch_lora_down(alch_dtype dt, const LoraDown* jobs, int n_jobs, int Trows, float alpha, long long ldy,
                     int slot_cols, hipStream_t stream) {
    if (n_jobs < 1 || n_jobs > 3) return fail(ALCH_ERR_INVALID_ARG, "adapter product: 1..3 problems per launch");
    double flops = 0, bytes = 0;
    bool fast = dt == ALCH_BF16;
    for (int i = 0; i < n_jobs; ++i) {
        const LoraDown& j = jobs[i];
        if (j.K % 8 || j.ldx % 8 || j.r % 8 || (j.r > 0 && j.lds % 8))
            return fail(ALCH_ERR_UNSUPPORTED, "adapter product: widths, strides and rank must be multiples of 8");
        if (j.r > 0) { flops += 2.0 * Trows * j.K * j.r; bytes += (double)Trows * j.K * dtype_size(dt); }
        fast = fast && j.K % 64 == 0 && aligned16(j.X) && (j.r == 0 || aligned16(j.S));
    }
    if (slot_cols % 8 || ldy % 8) return fail(ALCH_ERR_UNSUPPORTED, "adapter product: slot width must be a multiple of 8");
    if (Trows <= 0) return ALCH_OK;
    // algorithmic bytes: each streamed activation once (nothing for slots that are only zero-filled)
    TraceScope ts(kTraceLora, flops, bytes, stream);
    if (fast) {
        LoraDownParams p;
        for (int i = 0; i < 3; ++i) {
            const LoraDown& j = jobs[i < n_jobs ? i : 0];
            p.job[i] = LoraDownJob{(const __bf16*)j.X, j.ldx, j.K, (const __bf16*)j.S, j.lds, j.r, (__bf16*)j.Y};
        }
        p.Trows = Trows; p.ldy = ldy; p.alpha = alpha; p.slot_cols = slot_cols;
        k_lora_down_mfma<<<dim3(ceil_div(Trows, 32), ceil_div(slot_cols, 32), n_jobs), 256, 0, stream>>>(p);
    } else {
        for (int i = 0; i < n_jobs; ++i) {
            if (dt == ALCH_BF16) lora_down_valu<__bf16>(jobs[i], Trows, alpha, ldy, slot_cols, stream);
            else lora_down_valu<float>(jobs[i], Trows, alpha, ldy, slot_cols, stream);
        }
    }
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_lora_up(alch_dtype dt, const LoraUp* jobs, int n_jobs, int Trows, int r, float alpha, int accumulate,
                   float* scratch, hipStream_t stream) {
    if (n_jobs < 1 || n_jobs > kLoraUpJobs) return fail(ALCH_ERR_INVALID_ARG, "adapter gradient: 1..%d problems per launch", kLoraUpJobs);
    if (r % 8 || r <= 0) return fail(ALCH_ERR_UNSUPPORTED, "adapter gradient: rank must be a positive multiple of 8");
    LoraUpParams p;
    p.Trows = Trows; p.r = r; p.accumulate = accumulate; p.alpha = alpha; p.scratch = scratch;
    double flops = 0, bytes = 0;
    long long off = 0;
    int max_slabs = 1, max_split = 0, max_n = 1;
    for (int i = 0; i < kLoraUpJobs; ++i) {
        const LoraUp& j = jobs[i < n_jobs ? i : 0];
        if (i < n_jobs && (j.N % 8 || j.ldx % 8 || j.lds % 8))
            return fail(ALCH_ERR_UNSUPPORTED, "adapter gradient: widths and strides must be multiples of 8");
        const int nsplit = Trows > 0 ? up_splits(Trows, j.N) : 0;
        p.job[i] = LoraUpJob{j.S, j.lds, j.X, j.ldx, j.N, nsplit, nsplit > 0 ? ceil_div(Trows, nsplit) : 0, j.C, j.ldc, j.transposed, off};
        if (i < n_jobs) {
            off += (long long)(r / 8) * kLoraMaxSplits * 8 * j.N;  // the job's share of the scratch
            flops += 2.0 * Trows * j.N * r;
            bytes += (double)Trows * j.N * dtype_size(dt);
            max_slabs = std::max(max_slabs, ceil_div(j.N, 512));
            max_split = std::max(max_split, nsplit);
            max_n = std::max(max_n, j.N);
        }
    }
    TraceScope ts(kTraceLora, flops, bytes, stream);
    const dim3 grid_f(ceil_div((long long)max_n * r * 8, 256LL), n_jobs);
    if (dt == ALCH_BF16) {
        if (max_split > 0) k_lora_up_partial<__bf16><<<dim3(max_slabs, max_split, n_jobs * (r / 8)), 256, 0, stream>>>(p);
        k_lora_up_finish<__bf16><<<grid_f, 256, 0, stream>>>(p);
    } else {
        if (max_split > 0) k_lora_up_partial<float><<<dim3(max_slabs, max_split, n_jobs * (r / 8)), 256, 0, stream>>>(p);
        k_lora_up_finish<float><<<grid_f, 256, 0, stream>>>(p);
    }
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_lora_prep(alch_dtype dt, const LoraPrepParams& p, int n_jobs, hipStream_t stream) {
    if (n_jobs <= 0) return ALCH_OK;
    long long most = 0;
    for (int i = 0; i < n_jobs; ++i) most = std::max(most, (long long)p.job[i].rows_out * p.job[i].cols);
    int gx = ceil_div(most, 256LL);
    if (gx > 512) gx = 512;
    if (gx < 1) gx = 1;
    if (dt == ALCH_BF16) k_lora_prep<__bf16><<<dim3(gx, n_jobs), 256, 0, stream>>>(p);
    else k_lora_prep<float><<<dim3(gx, n_jobs), 256, 0, stream>>>(p);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
