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
// them.  A matrix-instruction operand wants one row per lane (a wave-wide load of that shape touches 64 cache
// lines for 1 KB); the rows are fetched as whole 128-byte lines straight into LDS instead (buffer_load ... lds,
// eight lanes per line) and the operands are read from there, which also lets several S share one pass over X.
//
// A problem = one streamed X [Trows, K] and up to four groups of eight columns of the output, each with its
// own [rows <= 8, K] matrix S and its own destination (problems that share X are merged by the host: the t1
// of q, k, v, or of gate and up, cost one pass).  A work-group owns 32 rows; its four wavefronts split K in
// chunks of 64 and fold their sums through LDS in a fixed order.  Every wavefront runs a private ring of
// stages [X 32 rows x 128 B | S 8 rows x 128 B per group]: no barrier inside the loop.  16-byte piece c of
// row r sits at position c ^ ((r >> 1) & 7) of the row, which makes the operand reads conflict-free.
typedef __attribute__((ext_vector_type(16))) float f32x16_l;
typedef __attribute__((ext_vector_type(4))) int i32x4_l;
struct LoraDownGroup {
    const __bf16* S; long long lds; int rows;  // rows = 0: no such group
    __bf16* Y;                                 // first of the group's eight output columns
};
static constexpr int kDownProblems = 6, kDownGroups = 4;
struct LoraDownProblem {
    const __bf16* X; long long ldx; int K, ngroups;
    LoraDownGroup g[kDownGroups];
};
struct LoraDownParams {
    LoraDownProblem pr[kDownProblems];
    __bf16* slot[3]; int slot_r[3]; int nslots;  // output slots: columns slot_r .. slot_cols-1 are zero-filled
    int Trows; long long ldy; float alpha; int slot_cols;
};
template <int kG> struct DownCfg {
    static constexpr int kStageBytes = 4096 + kG * 1024;
    static constexpr int kStages = kG == 1 ? 7 : kG == 2 ? 6 : kG == 3 ? 5 : 4;  // at most 36 KB per wavefront
};
__device__ __forceinline__ void lora_dma16(i32x4_l r, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(r)
                 : "memory", "m0");
}
__device__ __forceinline__ i32x4_l lora_rsrc(const void* p, long long bytes) {
    const uint32_t n = bytes <= 0 ? 0u : (bytes > 0x7fffffffLL ? 0x7fffffffu : (uint32_t)bytes);
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    i32x4_l r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)n);
    r[3] = 0x00020000;
    return r;
}
template <int kG>
__global__ __launch_bounds__(256) void k_lora_down_mfma(LoraDownParams p) {
    constexpr int kStageBytes = DownCfg<kG>::kStageBytes, kStages = DownCfg<kG>::kStages;
    __shared__ __attribute__((aligned(1024))) char smem[4 * kStages * kStageBytes];
    __shared__ float red[3][64][17];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 31, kh = lane >> 5;
    const long long t0 = (long long)blockIdx.x * 32;
    const int rows_valid = (int)(p.Trows - t0 < 32 ? p.Trows - t0 : 32);
    if (blockIdx.y == 0) {  // the columns past the rank of every output slot
        const int pieces = p.slot_cols >> 3;
        const bf16x8_l z = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
        for (int sl = 0; sl < p.nslots; ++sl)
            for (int idx = threadIdx.x; idx < 32 * pieces; idx += 256) {
                const int row = idx / pieces, piece = idx % pieces;
                if (row < rows_valid && piece * 8 >= p.slot_r[sl])
                    *reinterpret_cast<bf16x8_l*>(p.slot[sl] + (t0 + row) * p.ldy + piece * 8) = z;
            }
    }
    const LoraDownProblem& pb = p.pr[blockIdx.y];
    if (pb.ngroups == 0) return;
    const int nc = pb.K >> 6;
    const int c_lo = wave * nc / 4, n = (wave + 1) * nc / 4 - c_lo;  // this wavefront's chunks of 64 k
    char* wbase = smem + wave * (kStages * kStageBytes);
    const uint32_t lds_w = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) void*)wbase);
    // per-lane source offsets of the loads: lane -> (row 8j + lane/8, piece (lane & 7) ^ swizzle of the LDS row)
    const int row8 = lane >> 3, q = lane & 7;
    uint32_t voff_x[4], voff_s[kG];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + row8;
        voff_x[j] = (uint32_t)(row * pb.ldx * 2 + ((q ^ ((row >> 1) & 7)) << 4));
    }
#pragma unroll
    for (int g = 0; g < kG; ++g) voff_s[g] = (uint32_t)(row8 * pb.g[g].lds * 2 + ((q ^ (((8 * g + row8) >> 1) & 7)) << 4));
    const __bf16* xb = pb.X + t0 * pb.ldx + (long long)c_lo * 64;
    const long long x_bytes = rows_valid > 0 ? ((long long)(rows_valid - 1) * pb.ldx + 64) * 2 : 0;
    auto issue = [&](int i) {
        const uint32_t st = lds_w + (uint32_t)(i % kStages) * kStageBytes;
        const bool live = i < n;
        const i32x4_l rx = lora_rsrc(xb + (long long)i * 64, live ? x_bytes : 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) lora_dma16(rx, st + (uint32_t)j * 1024u, voff_x[j]);
#pragma unroll
        for (int g = 0; g < kG; ++g) {
            const LoraDownGroup& gr = pb.g[g];
            const i32x4_l rs = lora_rsrc(gr.S + (long long)(c_lo + i) * 64,
                                         live && gr.rows > 0 ? ((long long)(gr.rows - 1) * gr.lds + 64) * 2 : 0);
            lora_dma16(rs, st + 4096u + (uint32_t)g * 1024u, voff_s[g]);
        }
    };
    f32x16_l acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    // operand read offsets inside a stage: X row c, S row c (columns past the groups read a row that exists;
    // their results are never stored)
    const int cs = c < 8 * kG ? c : (c & 7);
    uint32_t off_a[4], off_b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        off_a[u] = (uint32_t)(c * 128 + (((2 * u + kh) ^ ((c >> 1) & 7)) << 4));
        off_b[u] = (uint32_t)(4096 + cs * 128 + (((2 * u + kh) ^ ((cs >> 1) & 7)) << 4));
    }
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s) issue(s);
    for (int i = 0; i < n; ++i) {
        issue(i + kStages - 1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 1) * (4 + kG)) : "memory");
        const char* st = wbase + (i % kStages) * kStageBytes;
        bf16x8_l a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = *reinterpret_cast<const bf16x8_l*>(st + off_a[u]);
            b[u] = *reinterpret_cast<const bf16x8_l*>(st + off_b[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u], acc, 0, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) red[wave - 1][lane][e] = acc[e];
    }
    __syncthreads();
    if (wave == 0) {
        __bf16* yp = nullptr;
        int yrows = 0;
#pragma unroll
        for (int g = 0; g < kG; ++g)
            if ((c >> 3) == g && g < pb.ngroups) { yp = pb.g[g].Y; yrows = pb.g[g].rows; }
        // accumulator element e: row 8*(e>>2) + 4*kh + (e&3), column c
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float v = ((acc[e] + red[0][lane][e]) + red[1][lane][e]) + red[2][lane][e];
            const int row = 8 * (e >> 2) + 4 * kh + (e & 3);
            if (row < rows_valid && (c & 7) < yrows) yp[(t0 + row) * p.ldy + (c & 7)] = (__bf16)(p.alpha * v);
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
        if (j.r > slot_cols) return fail(ALCH_ERR_INVALID_ARG, "adapter product: rank exceeds the output slot");
        fast = fast && j.K % 64 == 0 && aligned16(j.X) && aligned16(j.Y) && (j.r == 0 || aligned16(j.S)) && 32 * j.ldx < (1LL << 30);
    }
    if (slot_cols % 8 || ldy % 8) return fail(ALCH_ERR_UNSUPPORTED, "adapter product: slot width must be a multiple of 8");
    if (Trows <= 0) return ALCH_OK;
    // algorithmic bytes: each streamed activation once (nothing for slots that are only zero-filled)
    if (fast) {
        // problems: the eight-column groups of all jobs, those of equal X merged four at a time
        LoraDownParams p = {};
        int np = 0, most = 0;
        p.nslots = n_jobs;
        for (int i = 0; i < n_jobs; ++i) {
            const LoraDown& j = jobs[i];
            p.slot[i] = (__bf16*)j.Y;
            p.slot_r[i] = j.r;
            for (int g0 = 0; g0 < j.r; g0 += 8) {
                LoraDownProblem* pb = np > 0 ? &p.pr[np - 1] : nullptr;
                if (!pb || pb->X != (const __bf16*)j.X || pb->ldx != j.ldx || pb->K != j.K || pb->ngroups == kDownGroups) {
                    pb = &p.pr[np++];
                    pb->X = (const __bf16*)j.X; pb->ldx = j.ldx; pb->K = j.K; pb->ngroups = 0;
                }
                pb->g[pb->ngroups++] = LoraDownGroup{(const __bf16*)j.S + (long long)g0 * j.lds, j.lds, 8, (__bf16*)j.Y + g0};
                most = std::max(most, pb->ngroups);
            }
        }
        p.Trows = Trows; p.ldy = ldy; p.alpha = alpha; p.slot_cols = slot_cols;
        bytes = 0;
        for (int i = 0; i < np; ++i) bytes += (double)Trows * p.pr[i].K * dtype_size(dt);
        TraceScope ts(kTraceLora, flops, bytes, stream);
        const dim3 grid(ceil_div(Trows, 32), std::max(np, 1));
        if (most <= 1) k_lora_down_mfma<1><<<grid, 256, 0, stream>>>(p);
        else if (most == 2) k_lora_down_mfma<2><<<grid, 256, 0, stream>>>(p);
        else if (most == 3) k_lora_down_mfma<3><<<grid, 256, 0, stream>>>(p);
        else k_lora_down_mfma<4><<<grid, 256, 0, stream>>>(p);
    } else {
        TraceScope ts(kTraceLora, flops, bytes, stream);
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
