// Row-wise and elementwise kernels of the decoder-layer backward pass (RMSNorm forward and
// backward with the residual add, SwiGLU activation and its gradient, the softmax-gradient
// row term, rotary embedding).  All arithmetic in fp32; storage type T is float or bf16.
// These are HBM-bound: one pass over each operand, 16-byte accesses where alignment allows.
#include "kernels.h"

namespace alch {

template <typename T> __device__ __forceinline__ float ldf(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v) { *p = (T)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Sum over a 256-thread block (4 waves); every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float* smem /*[4]*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    return smem[0] + smem[1] + smem[2] + smem[3];
}

// ---- RMSNorm forward: H = X * rsqrt(mean(X^2) + eps) * g, one block per row
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm_fwd(const T* __restrict__ X, const T* __restrict__ g,
                                                     T* __restrict__ H, int width, float eps) {
    __shared__ float red[4];
    const long long row = blockIdx.x;
    const T* x = X + row * width;
    float ss = 0.f;
    for (int c = threadIdx.x; c < width; c += 256) {
        float v = ldf(x + c);
        ss += v * v;
    }
    ss = block_sum(ss, red);
    const float r = rsqrtf(ss / (float)width + eps);
    for (int c = threadIdx.x; c < width; c += 256) stf(H + row * width + c, ldf(x + c) * r * ldf(g + c));
}

// bf16 fast path: one wavefront per row, 16-byte accesses (lane l owns the 8-column chunks k*64 + l)
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_f;
template <int NC>
__global__ __launch_bounds__(256) void k_rmsnorm_fwd_bf16(const __bf16* __restrict__ X, const __bf16* __restrict__ g,
                                                          __bf16* __restrict__ H, int Trows, int width, float eps,
                                                          const int* __restrict__ rows_dev) {
    if (rows_dev) Trows = min(Trows, *rows_dev);  // row count decided on the device (compacted rows)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8_f gv[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        const int col = (k * 64 + lane) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) gv[k][e] = (__bf16)0.f;
        if (col < width) gv[k] = *reinterpret_cast<const bf16x8_f*>(g + col);
    }
    const float inv_w = 1.f / (float)width;
    for (long long row = (long long)blockIdx.x * 4 + wave; row < Trows; row += (long long)gridDim.x * 4) {
        bf16x8_f xv[NC];
        float ss = 0.f;
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int col = (k * 64 + lane) * 8;
            if (col < width) {
                xv[k] = *reinterpret_cast<const bf16x8_f*>(X + row * width + col);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += (float)xv[k][e] * (float)xv[k][e];
            }
        }
        ss = wave_sum(ss);
        const float r = rsqrtf(ss * inv_w + eps);
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int col = (k * 64 + lane) * 8;
            if (col < width) {
                bf16x8_f o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)xv[k][e] * r * (float)gv[k][e]);
                *reinterpret_cast<bf16x8_f*>(H + row * width + col) = o;
            }
        }
    }
}

int launch_rmsnorm_fwd(alch_dtype dt, const void* X, const void* g, void* H, int T, int width, float eps,
                       hipStream_t stream, const int* rows_dev) {
    if (T <= 0) return ALCH_OK;
    if (rows_dev && !(dt == ALCH_BF16 && width % 8 == 0 && width <= 8192 && aligned16(X) && aligned16(g) && aligned16(H)))
        return fail(ALCH_ERR_UNSUPPORTED, "device-side row count needs the bf16 row kernel");
    if (dt == ALCH_BF16 && width % 8 == 0 && width <= 8192 && aligned16(X) && aligned16(g) && aligned16(H)) {
        const int nblk = ceil_div(T, 4) < 2048 ? ceil_div(T, 4) : 2048;
#define ALCH_NORM_FWD(NC) \
    k_rmsnorm_fwd_bf16<NC><<<nblk, 256, 0, stream>>>((const __bf16*)X, (const __bf16*)g, (__bf16*)H, T, width, eps, rows_dev)
        if (width <= 1024) ALCH_NORM_FWD(2);
        else if (width <= 2048) ALCH_NORM_FWD(4);
        else if (width <= 4096) ALCH_NORM_FWD(8);
        else ALCH_NORM_FWD(16);
#undef ALCH_NORM_FWD
        ALCH_HIP_TRY(hipGetLastError());
        return ALCH_OK;
    }
    if (dt == ALCH_BF16)
        k_rmsnorm_fwd<__bf16><<<T, 256, 0, stream>>>((const __bf16*)X, (const __bf16*)g, (__bf16*)H, width, eps);
    else
        k_rmsnorm_fwd<float><<<T, 256, 0, stream>>>((const float*)X, (const float*)g, (float*)H, width, eps);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// ---- RMSNorm backward with residual:
//   dX = resid + r*(g*dH) - X * r^3/width * sum(g*dH*X);   dg partial[blk] = sum over the block's rows of dH*X*r
static constexpr int kNormBwdBlocks = 1024;
static constexpr int kNormMaxCols = 32;  // columns per thread: width <= 8192

int rmsnorm_bwd_blocks(int T);

template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm_bwd(const T* __restrict__ dH, const T* __restrict__ X,
                                                     const T* __restrict__ g, const T* __restrict__ resid,
                                                     const uint8_t* __restrict__ resid_mask, T* __restrict__ dX,
                                                     float* __restrict__ partial, int Trows, int width, float eps) {
    __shared__ float red[4];
    float dgp[kNormMaxCols];
    float gv[kNormMaxCols];
#pragma unroll
    for (int i = 0; i < kNormMaxCols; ++i) {
        dgp[i] = 0.f;
        const int c = threadIdx.x + 256 * i;
        gv[i] = c < width ? ldf(g + c) : 0.f;
    }
    for (long long row = blockIdx.x; row < Trows; row += gridDim.x) {
        float xv[kNormMaxCols], dv[kNormMaxCols];
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int i = 0; i < kNormMaxCols; ++i) {
            const int c = threadIdx.x + 256 * i;
            xv[i] = c < width ? ldf(X + row * width + c) : 0.f;
            dv[i] = c < width ? ldf(dH + row * width + c) : 0.f;
            ss += xv[i] * xv[i];
            dot += gv[i] * dv[i] * xv[i];
        }
        ss = block_sum(ss, red);
        dot = block_sum(dot, red);
        const float r = rsqrtf(ss / (float)width + eps);
        const float coef = r * r * r / (float)width * dot;
        const bool keep = resid && !(resid_mask && resid_mask[row] == 0);
#pragma unroll
        for (int i = 0; i < kNormMaxCols; ++i) {
            const int c = threadIdx.x + 256 * i;
            if (c < width) {
                float v = r * gv[i] * dv[i] - xv[i] * coef;
                if (keep) v += ldf(resid + row * width + c);
                stf(dX + row * width + c, v);
                dgp[i] += dv[i] * xv[i] * r;
            }
        }
    }
    if (partial) {
#pragma unroll
        for (int i = 0; i < kNormMaxCols; ++i) {
            const int c = threadIdx.x + 256 * i;
            if (c < width) partial[(long long)blockIdx.x * width + c] = dgp[i];
        }
    }
}

// bf16 fast path: one wavefront per row, 16-byte accesses, no barrier inside the row loop.
// Lane l owns the 8-column chunks (k*64 + l), k < NC.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
static constexpr int kNormFastBlocks = 512;

template <int NC>
__global__ __launch_bounds__(256) void k_rmsnorm_bwd_bf16(const __bf16* __restrict__ dH, const __bf16* __restrict__ X,
                                                          const __bf16* __restrict__ g, const __bf16* __restrict__ resid,
                                                          const uint8_t* __restrict__ resid_mask, __bf16* __restrict__ dX,
                                                          float* __restrict__ partial, int Trows, int width, float eps,
                                                          const int* __restrict__ rows_dev, __bf16* __restrict__ hn_out) {
    __shared__ float sred[NC * 512];
    if (rows_dev) Trows = min(Trows, *rows_dev);  // row count decided on the device (compacted rows)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8_t gv[NC];
    float dgp[NC][8];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        const int col = (k * 64 + lane) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { gv[k][e] = (__bf16)0.f; dgp[k][e] = 0.f; }
        if (col < width) gv[k] = *reinterpret_cast<const bf16x8_t*>(g + col);
    }
    const float inv_w = 1.f / (float)width;
    for (long long row = (long long)blockIdx.x * 4 + wave; row < Trows; row += (long long)gridDim.x * 4) {
        bf16x8_t xv[NC], dv[NC];
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int col = (k * 64 + lane) * 8;
            if (col < width) {
                xv[k] = *reinterpret_cast<const bf16x8_t*>(X + row * width + col);
                dv[k] = *reinterpret_cast<const bf16x8_t*>(dH + row * width + col);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) { xv[k][e] = (__bf16)0.f; dv[k][e] = (__bf16)0.f; }
            }
        }
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int k = 0; k < NC; ++k)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = (float)xv[k][e];
                ss += x * x;
                dot += (float)gv[k][e] * (float)dv[k][e] * x;
            }
        ss = wave_sum(ss);
        dot = wave_sum(dot);
        const float r = rsqrtf(ss * inv_w + eps);
        const float coef = r * r * r * inv_w * dot;
        const bool keep = resid && !(resid_mask && resid_mask[row] == 0);
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int col = (k * 64 + lane) * 8;
            if (col < width) {
                bf16x8_t rv, ov;
                if (keep) rv = *reinterpret_cast<const bf16x8_t*>(resid + row * width + col);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = (float)xv[k][e], d = (float)dv[k][e];
                    float v = r * (float)gv[k][e] * d - x * coef;
                    if (keep) v += (float)rv[e];
                    ov[e] = (__bf16)v;
                    dgp[k][e] += d * x * r;
                }
                *reinterpret_cast<bf16x8_t*>(dX + row * width + col) = ov;
                if (hn_out) {  // the normalised row itself (the forward's value), for the weight gradients that follow
                    bf16x8_t hv;
#pragma unroll
                    for (int e = 0; e < 8; ++e) hv[e] = (__bf16)((float)xv[k][e] * r * (float)gv[k][e]);
                    *reinterpret_cast<bf16x8_t*>(hn_out + row * width + col) = hv;
                }
            }
        }
    }
    if (!partial) return;
    // fold the four waves' column sums in a fixed order, then one row of partials per block
    for (int w = 1; w < 4; ++w) {
        __syncthreads();
        if (wave == w)
#pragma unroll
            for (int k = 0; k < NC; ++k)
#pragma unroll
                for (int e = 0; e < 8; ++e) sred[(k * 8 + e) * 64 + lane] = dgp[k][e];
        __syncthreads();
        if (wave == 0)
#pragma unroll
            for (int k = 0; k < NC; ++k)
#pragma unroll
                for (int e = 0; e < 8; ++e) dgp[k][e] += sred[(k * 8 + e) * 64 + lane];
    }
    if (wave == 0)
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int col = (k * 64 + lane) * 8;
            if (col < width)
#pragma unroll
                for (int e = 0; e < 8; ++e) partial[(long long)blockIdx.x * width + col + e] = dgp[k][e];
        }
}

// dg[c] (+)= sum over nblk partial rows; 64 columns per block, 16 row groups folded through LDS
template <typename T>
__global__ __launch_bounds__(1024) void k_colsum_finish_wide(const float* __restrict__ partial, int nblk, int width,
                                                             T* __restrict__ dg, int accumulate) {
    __shared__ float red[16][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63), rg = threadIdx.x >> 6;
    float s = 0.f;
    if (c < width)
        for (int b = rg; b < nblk; b += 16) s += partial[(long long)b * width + c];
    red[rg][threadIdx.x & 63] = s;
    __syncthreads();
    if (rg == 0 && c < width) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) t += red[i][threadIdx.x & 63];
        if (accumulate) t += ldf(dg + c);
        stf(dg + c, t);
    }
}

int rmsnorm_bwd_blocks(int T) {
    const int n = T < kNormBwdBlocks ? (T > 0 ? T : 1) : kNormBwdBlocks;
    return n > kNormFastBlocks ? n : kNormFastBlocks;  // scratch rows: enough for either kernel
}

template <typename T>
static int rmsnorm_bwd_t(const void* dH, const void* X, const void* g, const void* resid, const uint8_t* resid_mask,
                         void* dX, void* dg, int accumulate, float* partial, int T_, int width, float eps,
                         hipStream_t stream) {
    const int nblk = T_ < kNormBwdBlocks ? T_ : kNormBwdBlocks;
    k_rmsnorm_bwd<T><<<nblk, 256, 0, stream>>>((const T*)dH, (const T*)X, (const T*)g, (const T*)resid, resid_mask,
                                                (T*)dX, dg ? partial : nullptr, T_, width, eps);
    if (dg) k_colsum_finish_wide<T><<<ceil_div(width, 64), 1024, 0, stream>>>(partial, nblk, width, (T*)dg, accumulate);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// Wide rows (width > 2048): WPR wavefronts share a row, each owning a quarter or half of its columns (4 chunks of
// 8 per lane), so the per-lane state stays small enough for several wavefronts per SIMD; the two row sums meet
// through LDS in wavefront order.  Every wavefront runs the same number of iterations (barriers inside).
template <int WPR>
__global__ __launch_bounds__(256) void k_rmsnorm_bwd_bf16_split(const __bf16* __restrict__ dH, const __bf16* __restrict__ X,
                                                                const __bf16* __restrict__ g, const __bf16* __restrict__ resid,
                                                                const uint8_t* __restrict__ resid_mask,
                                                                __bf16* __restrict__ dX, float* __restrict__ partial,
                                                                int Trows, int width, float eps,
                                                                const int* __restrict__ rows_dev, __bf16* __restrict__ hn_out) {
    constexpr int RPB = 4 / WPR;  // rows per work-group per iteration
    __shared__ float rsum[2][4][2];
    __shared__ float sred[2 * 4 * 8 * 64];  // [part][chunk][element][lane], used when two rows share a work-group
    if (rows_dev) Trows = min(Trows, *rows_dev);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int part = wave % WPR, rsel = wave / WPR;
    bf16x8_t gv[4];
    float dgp[4][8];
    int col[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        col[k] = ((k * WPR + part) * 64 + lane) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { gv[k][e] = (__bf16)0.f; dgp[k][e] = 0.f; }
        if (col[k] < width) gv[k] = *reinterpret_cast<const bf16x8_t*>(g + col[k]);
    }
    const float inv_w = 1.f / (float)width;
    const long long stride = (long long)gridDim.x * RPB;
    const int iters = (int)((Trows + stride - 1) / stride);
    for (int it = 0; it < iters; ++it) {
        const long long row = (long long)it * stride + (long long)blockIdx.x * RPB + rsel;
        const bool live = row < Trows;
        const bool keep = live && resid && !(resid_mask && resid_mask[row] == 0);
        bf16x8_t xv[4], dv[4], rv[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { xv[k][e] = (__bf16)0.f; dv[k][e] = (__bf16)0.f; rv[k][e] = (__bf16)0.f; }
            if (live && col[k] < width) {
                xv[k] = *reinterpret_cast<const bf16x8_t*>(X + row * width + col[k]);
                dv[k] = *reinterpret_cast<const bf16x8_t*>(dH + row * width + col[k]);
                if (keep) rv[k] = *reinterpret_cast<const bf16x8_t*>(resid + row * width + col[k]);
            }
        }
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = (float)xv[k][e];
                ss += x * x;
                dot += (float)gv[k][e] * (float)dv[k][e] * x;
            }
        ss = wave_sum(ss);
        dot = wave_sum(dot);
        if (WPR > 1) {
            if (lane == 0) { rsum[it & 1][wave][0] = ss; rsum[it & 1][wave][1] = dot; }
            __syncthreads();
            ss = 0.f; dot = 0.f;
#pragma unroll
            for (int w = 0; w < WPR; ++w) { ss += rsum[it & 1][rsel * WPR + w][0]; dot += rsum[it & 1][rsel * WPR + w][1]; }
        }
        const float r = rsqrtf(ss * inv_w + eps);
        const float coef = r * r * r * inv_w * dot;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (live && col[k] < width) {
                bf16x8_t ov;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = (float)xv[k][e], d = (float)dv[k][e];
                    const float v = r * (float)gv[k][e] * d - x * coef + (float)rv[k][e];
                    ov[e] = (__bf16)v;
                    dgp[k][e] += d * x * r;
                }
                *reinterpret_cast<bf16x8_t*>(dX + row * width + col[k]) = ov;
                if (hn_out) {  // the normalised row itself (the forward's value), for the weight gradients that follow
                    bf16x8_t hv;
#pragma unroll
                    for (int e = 0; e < 8; ++e) hv[e] = (__bf16)((float)xv[k][e] * r * (float)gv[k][e]);
                    *reinterpret_cast<bf16x8_t*>(hn_out + row * width + col[k]) = hv;
                }
            }
        }
    }
    if (!partial) return;
    // column sums: the RPB wavefronts that own the same columns fold theirs in a fixed order
    for (int rs = 1; rs < RPB; ++rs) {
        __syncthreads();
        if (rsel == rs)
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int e = 0; e < 8; ++e) sred[((part * 4 + k) * 8 + e) * 64 + lane] = dgp[k][e];
        __syncthreads();
        if (rsel == 0)
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int e = 0; e < 8; ++e) dgp[k][e] += sred[((part * 4 + k) * 8 + e) * 64 + lane];
    }
    if (rsel == 0)
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (col[k] < width)
#pragma unroll
                for (int e = 0; e < 8; ++e) partial[(long long)blockIdx.x * width + col[k] + e] = dgp[k][e];
}

static int rmsnorm_bwd_bf16_fast(const void* dH, const void* X, const void* g, const void* resid,
                                 const uint8_t* resid_mask, void* dX, void* dg, int accumulate, float* partial, int T_,
                                 int width, float eps, hipStream_t stream, const int* rows_dev, void* hn_out) {
    const int nblk = ceil_div(T_, 4) < kNormFastBlocks ? ceil_div(T_, 4) : kNormFastBlocks;
    float* part = dg ? partial : nullptr;
#define ALCH_NORM_BWD(NC)                                                                                          \
    k_rmsnorm_bwd_bf16<NC><<<nblk, 256, 0, stream>>>((const __bf16*)dH, (const __bf16*)X, (const __bf16*)g,         \
                                                     (const __bf16*)resid, resid_mask, (__bf16*)dX, part, T_, width, eps, rows_dev, (__bf16*)hn_out)
#define ALCH_NORM_BWD_SPLIT(WPR)                                                                                    \
    k_rmsnorm_bwd_bf16_split<WPR><<<nblk, 256, 0, stream>>>((const __bf16*)dH, (const __bf16*)X, (const __bf16*)g,  \
                                                            (const __bf16*)resid, resid_mask, (__bf16*)dX, part, T_, width, eps, rows_dev, (__bf16*)hn_out)
    if (width <= 1024) ALCH_NORM_BWD(2);
    else if (width <= 2048) ALCH_NORM_BWD(4);
    else if (width <= 4096) ALCH_NORM_BWD_SPLIT(2);
    else ALCH_NORM_BWD_SPLIT(4);
#undef ALCH_NORM_BWD
#undef ALCH_NORM_BWD_SPLIT
    if (dg) k_colsum_finish_wide<__bf16><<<ceil_div(width, 64), 1024, 0, stream>>>(partial, nblk, width, (__bf16*)dg, accumulate);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_rmsnorm_bwd(alch_dtype dt, const void* dH, const void* X, const void* g, const void* resid,
                       const uint8_t* resid_mask, void* dX, void* dg, int accumulate, float* partial, int T,
                       int width, float eps, hipStream_t stream, const int* rows_dev, void* hn_out) {
    if (width > 256 * kNormMaxCols) return fail(ALCH_ERR_UNSUPPORTED, "hidden %d > %d", width, 256 * kNormMaxCols);
    if (T <= 0) {
        // no rows: the gain gradient is zero (or unchanged when accumulating)
        if (dg) {
            if (dt == ALCH_BF16)
                k_colsum_finish_wide<__bf16><<<ceil_div(width, 64), 1024, 0, stream>>>(partial, 0, width, (__bf16*)dg, accumulate);
            else
                k_colsum_finish_wide<float><<<ceil_div(width, 64), 1024, 0, stream>>>(partial, 0, width, (float*)dg, accumulate);
            ALCH_HIP_TRY(hipGetLastError());
        }
        return ALCH_OK;
    }
    if (dt == ALCH_BF16 && width % 8 == 0 && aligned16(dH) && aligned16(X) && aligned16(g) && aligned16(dX) &&
        (!resid || aligned16(resid)) && (!hn_out || (aligned16(hn_out) && hn_out != dX)))
        return rmsnorm_bwd_bf16_fast(dH, X, g, resid, resid_mask, dX, dg, accumulate, partial, T, width, eps, stream, rows_dev, hn_out);
    if (rows_dev) return fail(ALCH_ERR_UNSUPPORTED, "device-side row count needs the bf16 row kernel");
    if (hn_out) ALCH_TRY(launch_rmsnorm_fwd(dt, X, g, hn_out, T, width, eps, stream));  // plain kernels: the forward's own kernel
    return dt == ALCH_BF16
               ? rmsnorm_bwd_t<__bf16>(dH, X, g, resid, resid_mask, dX, dg, accumulate, partial, T, width, eps, stream)
               : rmsnorm_bwd_t<float>(dH, X, g, resid, resid_mask, dX, dg, accumulate, partial, T, width, eps, stream);
}

// ---- SwiGLU
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu_act(const T* __restrict__ G, const T* __restrict__ U,
                                                    T* __restrict__ Act, long long n) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const float g = ldf(G + i), u = ldf(U + i);
        stf(Act + i, g / (1.f + __expf(-g)) * u);
    }
}

// bf16, 8 elements per thread (n a multiple of 8, 16-byte aligned operands)
__global__ __launch_bounds__(256) void k_swiglu_act_bf16x8(const bf16x8_t* __restrict__ G, const bf16x8_t* __restrict__ U,
                                                           bf16x8_t* __restrict__ Act, long long n8) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        const bf16x8_t g = __builtin_nontemporal_load(G + i), u = __builtin_nontemporal_load(U + i);
        bf16x8_t a;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float gf = (float)g[e];
            a[e] = (__bf16)(gf / (1.f + __expf(-gf)) * (float)u[e]);
        }
        Act[i] = a;
    }
}

int launch_swiglu_act(alch_dtype dt, const void* G, const void* U, void* Act, long long n, hipStream_t stream) {
    if (n <= 0) return ALCH_OK;
    if (dt == ALCH_BF16 && n % 8 == 0 && aligned16(G) && aligned16(U) && aligned16(Act)) {
        const long long n8 = n / 8;
        const int grid8 = (int)((n8 + 255) / 256 < 256 * 32 ? (n8 + 255) / 256 : 256 * 32);
        k_swiglu_act_bf16x8<<<grid8, 256, 0, stream>>>((const bf16x8_t*)G, (const bf16x8_t*)U, (bf16x8_t*)Act, n8);
        ALCH_HIP_TRY(hipGetLastError());
        return ALCH_OK;
    }
    const int grid = (int)((n + 255) / 256 < 256 * 16 ? (n + 255) / 256 : 256 * 16);
    if (dt == ALCH_BF16)
        k_swiglu_act<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)G, (const __bf16*)U, (__bf16*)Act, n);
    else
        k_swiglu_act<float><<<grid, 256, 0, stream>>>((const float*)G, (const float*)U, (float*)Act, n);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

template <typename T>
__global__ __launch_bounds__(256) void k_swiglu_bwd(const T* __restrict__ dAct, const T* __restrict__ G,
                                                    const T* __restrict__ U, T* __restrict__ dGU,
                                                    T* __restrict__ Act, int Trows, int F) {
    const long long n = (long long)Trows * F;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const long long t = i / F;
        const int f = (int)(i - t * F);
        const float g = ldf(G + i), u = ldf(U + i), d = ldf(dAct + i);
        const float sg = 1.f / (1.f + __expf(-g));
        stf(dGU + t * 2 * F + f, d * u * sg * (1.f + g * (1.f - sg)));
        stf(dGU + t * 2 * F + F + f, d * g * sg);
        if (Act) stf(Act + i, g * sg * u);
    }
}

int launch_swiglu_bwd(alch_dtype dt, const void* dAct, const void* G, const void* U, void* dGU, void* Act, int T,
                      int F, hipStream_t stream) {
    const long long n = (long long)T * F;
    if (n <= 0) return ALCH_OK;
    const int grid = (int)((n + 255) / 256 < 256 * 16 ? (n + 255) / 256 : 256 * 16);
    if (dt == ALCH_BF16)
        k_swiglu_bwd<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)dAct, (const __bf16*)G, (const __bf16*)U,
                                                       (__bf16*)dGU, (__bf16*)Act, T, F);
    else
        k_swiglu_bwd<float><<<grid, 256, 0, stream>>>((const float*)dAct, (const float*)G, (const float*)U,
                                                      (float*)dGU, (float*)Act, T, F);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// ---- delta[t,h] = sum_d dO*O : one wave per (t,h)
template <typename T>
__global__ __launch_bounds__(256) void k_attn_delta(const T* __restrict__ dO, const T* __restrict__ O,
                                                    float* __restrict__ delta, long long n_rows, int D) {
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    for (int d = lane; d < D; d += 64) s += ldf(dO + row * D + d) * ldf(O + row * D + d);
    s = wave_sum(s);
    if (lane == 0) delta[row] = s;
}

int launch_attn_delta(alch_dtype dt, const void* dO, const void* O, float* delta, int T, int Hq, int D,
                      hipStream_t stream) {
    const long long n = (long long)T * Hq;
    if (n <= 0) return ALCH_OK;
    const int grid = (int)((n + 3) / 4);
    if (dt == ALCH_BF16)
        k_attn_delta<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)dO, (const __bf16*)O, delta, n, D);
    else
        k_attn_delta<float><<<grid, 256, 0, stream>>>((const float*)dO, (const float*)O, delta, n, D);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// ---- rotary embedding in place: pairs (i, i + D/2), angle = pos * base^(-2i/D), rotation by sign*angle
template <typename T>
__global__ __launch_bounds__(256) void k_rope(T* __restrict__ x, long long ld, int Trows, int n_heads, int D,
                                              const int* __restrict__ positions, const int* __restrict__ cu_seqlens,
                                              int n_seqs, float log2_base, float sign) {
    const int half = D >> 1;
    const long long per_row = (long long)n_heads * half;
    const long long n = (long long)Trows * per_row;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const long long t = i / per_row;
        const int rem = (int)(i - t * per_row);
        const int h = rem / half, k = rem - h * half;
        int pos;
        if (positions) {
            pos = positions[t];
        } else {
            // binary search for the sequence that holds token t
            int lo = 0, hi = n_seqs;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (cu_seqlens[mid] <= t) lo = mid; else hi = mid;
            }
            pos = (int)t - cu_seqlens[lo];
        }
        const float theta = exp2f(-2.f * (float)k / (float)D * log2_base);
        float sn, cs;
        sincosf((float)pos * theta, &sn, &cs);
        sn *= sign;
        T* p = x + t * ld + (long long)h * D + k;
        const float a = ldf(p), b = ldf(p + half);
        stf(p, a * cs - b * sn);
        stf(p + half, b * cs + a * sn);
    }
}

// bf16, head_dim a multiple of 16: a thread owns 8 consecutive pairs of one token, computes their sines and
// cosines once and applies them to every kHeadLanes-th head (all heads of a token share the angles).
static constexpr int kHeadLanes = 8;
__global__ __launch_bounds__(256) void k_rope_bf16x8(__bf16* __restrict__ x, long long ld, int Trows, int n_heads, int D,
                                                     const int* __restrict__ positions, const int* __restrict__ cu_seqlens,
                                                     int n_seqs, float log2_base, float sign) {
    const int half = D >> 1, kc = half >> 3;  // 8-pair chunks per head
    const int per_tok = kc * kHeadLanes;
    const long long n = (long long)Trows * per_tok;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const long long t = i / per_tok;
        const int rem = (int)(i - t * per_tok);
        const int hl = rem / kc, k0 = (rem - hl * kc) * 8;
        if (hl >= n_heads) continue;
        int pos;
        if (positions) {
            pos = positions[t];
        } else {
            int lo = 0, hi = n_seqs;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (cu_seqlens[mid] <= t) lo = mid; else hi = mid;
            }
            pos = (int)t - cu_seqlens[lo];
        }
        float sn[8], cs[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float theta = exp2f(-2.f * (float)(k0 + e) / (float)D * log2_base);
            sincosf((float)pos * theta, &sn[e], &cs[e]);
            sn[e] *= sign;
        }
        for (int h = hl; h < n_heads; h += kHeadLanes) {
            __bf16* p = x + t * ld + (long long)h * D + k0;
            const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(p), b = *reinterpret_cast<const bf16x8_t*>(p + half);
            bf16x8_t ra, rb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float af = (float)a[e], bf = (float)b[e];
                ra[e] = (__bf16)(af * cs[e] - bf * sn[e]);
                rb[e] = (__bf16)(bf * cs[e] + af * sn[e]);
            }
            *reinterpret_cast<bf16x8_t*>(p) = ra;
            *reinterpret_cast<bf16x8_t*>(p + half) = rb;
        }
    }
}

int launch_rope(alch_dtype dt, void* x, long long ld, int T, int n_heads, int D, const int* positions,
                const int* cu_seqlens, int n_seqs, float base, float sign, hipStream_t stream) {
    const long long n = (long long)T * n_heads * (D / 2);
    if (n <= 0) return ALCH_OK;
    if (dt == ALCH_BF16 && D % 16 == 0 && ld % 8 == 0 && aligned16(x)) {
        const long long nt = (long long)T * (D / 16) * kHeadLanes;
        const int g = (int)((nt + 255) / 256 < 256 * 32 ? (nt + 255) / 256 : 256 * 32);
        k_rope_bf16x8<<<g, 256, 0, stream>>>((__bf16*)x, ld, T, n_heads, D, positions, cu_seqlens, n_seqs, log2f(base), sign);
        ALCH_HIP_TRY(hipGetLastError());
        return ALCH_OK;
    }
    const int grid = (int)((n + 255) / 256 < 256 * 16 ? (n + 255) / 256 : 256 * 16);
    const float l2 = log2f(base);
    if (dt == ALCH_BF16)
        k_rope<__bf16><<<grid, 256, 0, stream>>>((__bf16*)x, ld, T, n_heads, D, positions, cu_seqlens, n_seqs, l2, sign);
    else
        k_rope<float><<<grid, 256, 0, stream>>>((float*)x, ld, T, n_heads, D, positions, cu_seqlens, n_seqs, l2, sign);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// ---- masked copy / add
template <typename T>
__global__ __launch_bounds__(256) void k_masked_copy(const T* __restrict__ a, const uint8_t* __restrict__ mask,
                                                     T* __restrict__ out, int Trows, int width) {
    const long long n = (long long)Trows * width;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const long long t = i / width;
        out[i] = (mask && mask[t] == 0) ? (T)0.f : a[i];
    }
}

// 16 bytes per thread; `per_row` = 16-byte chunks in a row (the row bytes are a multiple of 16)
__global__ __launch_bounds__(256) void k_masked_copy_x16(const uint4* __restrict__ a, const uint8_t* __restrict__ mask,
                                                         uint4* __restrict__ out, long long n16, int per_row) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long long)gridDim.x * 256) {
        uint4 v = a[i];
        if (mask && mask[i / per_row] == 0) v = make_uint4(0u, 0u, 0u, 0u);
        out[i] = v;
    }
}

int launch_masked_copy(alch_dtype dt, const void* a, const uint8_t* mask, void* out, int T, int width,
                       hipStream_t stream) {
    const long long n = (long long)T * width;
    if (n <= 0) return ALCH_OK;
    const long long row_bytes = (long long)width * (long long)dtype_size(dt);
    if (row_bytes % 16 == 0 && aligned16(a) && aligned16(out)) {
        const long long n16 = (long long)T * (row_bytes / 16);
        const int g = (int)((n16 + 255) / 256 < 256 * 32 ? (n16 + 255) / 256 : 256 * 32);
        k_masked_copy_x16<<<g, 256, 0, stream>>>((const uint4*)a, mask, (uint4*)out, n16, (int)(row_bytes / 16));
        ALCH_HIP_TRY(hipGetLastError());
        return ALCH_OK;
    }
    const int grid = (int)((n + 255) / 256 < 256 * 16 ? (n + 255) / 256 : 256 * 16);
    if (dt == ALCH_BF16)
        k_masked_copy<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)a, mask, (__bf16*)out, T, width);
    else
        k_masked_copy<float><<<grid, 256, 0, stream>>>((const float*)a, mask, (float*)out, T, width);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

template <typename T>
__global__ __launch_bounds__(256) void k_add(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ y,
                                             long long n) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
        stf(y + i, ldf(a + i) + ldf(b + i));
}

int launch_add(alch_dtype dt, const void* a, const void* b, void* y, long long n, hipStream_t stream) {
    if (n <= 0) return ALCH_OK;
    const int grid = (int)((n + 255) / 256 < 256 * 16 ? (n + 255) / 256 : 256 * 16);
    if (dt == ALCH_BF16)
        k_add<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)a, (const __bf16*)b, (__bf16*)y, n);
    else
        k_add<float><<<grid, 256, 0, stream>>>((const float*)a, (const float*)b, (float*)y, n);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

// ---- row scatter: out [T, width] = src[rank of t among the kept rows, :] for kept t, zeros elsewhere.
// inv[t] = that rank or -1 is built first (two launches: clear, then fill from the kept-row index), so the
// scatter writes every row of `out` exactly once, 16 bytes per lane.
__global__ __launch_bounds__(256) void k_rank_clear(int* __restrict__ inv, int T_) {
    for (int i = blockIdx.x * 256 + threadIdx.x; i < T_; i += gridDim.x * 256) inv[i] = -1;
}
__global__ __launch_bounds__(256) void k_rank_fill(const int* __restrict__ index, const int* __restrict__ n_rows,
                                                   int* __restrict__ inv, int T_) {
    const int n = min(*n_rows, T_);
    for (int r = blockIdx.x * 256 + threadIdx.x; r < n; r += gridDim.x * 256) inv[index[r]] = r;
}
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__global__ __launch_bounds__(256) void k_scatter_rows(const u32x4_t* __restrict__ src, const int* __restrict__ inv,
                                                      u32x4_t* __restrict__ out, int T_, int pieces) {
    for (int t = blockIdx.x; t < T_; t += gridDim.x) {
        const int r = inv[t];
        for (int c = threadIdx.x; c < pieces; c += 256) {
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (r >= 0) v = src[(long long)r * pieces + c];
            out[(long long)t * pieces + c] = v;
        }
    }
}

int launch_rank_of_kept(const int* index, const int* n_rows, int* inv, int T_, hipStream_t stream) {
    if (T_ <= 0) return ALCH_OK;
    const int nb = ceil_div(T_, 256) < 1024 ? ceil_div(T_, 256) : 1024;
    k_rank_clear<<<nb, 256, 0, stream>>>(inv, T_);
    k_rank_fill<<<nb, 256, 0, stream>>>(index, n_rows, inv, T_);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_scatter_rows(const void* src, const int* inv, void* out, int T_, size_t row_bytes, hipStream_t stream) {
    if (T_ <= 0) return ALCH_OK;
    if (row_bytes % 16 || !aligned16(src) || !aligned16(out)) return fail(ALCH_ERR_UNSUPPORTED, "scatter: rows must be 16-byte multiples");
    k_scatter_rows<<<T_ < 65536 ? T_ : 65536, 256, 0, stream>>>((const u32x4_t*)src, inv, (u32x4_t*)out, T_, (int)(row_bytes / 16));
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
