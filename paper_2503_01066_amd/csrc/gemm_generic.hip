// Plain tiled GEMM in fp32 arithmetic for the fp32 storage type and for bf16 problems whose
// shapes or alignments the matrix-core kernel does not take.  Same contract as the
// matrix-core kernel (segments, split outputs, accumulate); correctness first.
#include "kernels.h"
#include <hip/hip_bf16.h>

namespace alch {

struct GenericGemmParams {
    int M, N, n_seg, n_out, accumulate, a_kmajor, b_kmajor;
    const void* A[kMaxGemmSegs];
    const void* B[kMaxGemmSegs];
    int K[kMaxGemmSegs];
    long long lda[kMaxGemmSegs], ldb[kMaxGemmSegs];
    void* C[3];
    int m_begin[3];
    long long ldc[3];
    int epilogue;
    const void* G;
    const void* U;
    long long ldgu;
    void* act_out;
    const uint8_t* row_mask;
};

template <typename T> __device__ __forceinline__ float ld(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void st(T* p, float v) { *p = (T)v; }

template <typename T>
__global__ __launch_bounds__(256) void k_gemm_generic(GenericGemmParams p) {
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 1];
    __shared__ float Bs[TK][TN + 1];
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int s = 0; s < p.n_seg; ++s) {
        const T* A = static_cast<const T*>(p.A[s]);
        const T* B = static_cast<const T*>(p.B[s]);
        const long long lda = p.lda[s], ldb = p.ldb[s];
        const int K = p.K[s];
        for (int k0 = 0; k0 < K; k0 += TK) {
            for (int e = threadIdx.x; e < TM * TK; e += 256) {
                int mm, kk;
                if (p.a_kmajor) { mm = e / TK; kk = e % TK; } else { kk = e / TM; mm = e % TM; }
                const int m = m0 + mm, k = k0 + kk;
                float v = 0.f;
                if (m < p.M && k < K && !(p.row_mask && p.row_mask[m] == 0))
                    v = ld(p.a_kmajor ? A + (long long)m * lda + k : A + (long long)k * lda + m);
                As[kk][mm] = v;
            }
            for (int e = threadIdx.x; e < TN * TK; e += 256) {
                int nn, kk;
                if (p.b_kmajor) { nn = e / TK; kk = e % TK; } else { kk = e / TN; nn = e % TN; }
                const int n = n0 + nn, k = k0 + kk;
                float v = 0.f;
                if (n < p.N && k < K) v = ld(p.b_kmajor ? B + (long long)n * ldb + k : B + (long long)k * ldb + n);
                Bs[kk][nn] = v;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < TK; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx + 16 * j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        if (m >= p.M) continue;
        int oseg = 0;
        for (int s = 1; s < p.n_out; ++s)
            if (m >= p.m_begin[s]) oseg = s;
        T* C = static_cast<T*>(p.C[oseg]);
        const long long ldc = p.ldc[oseg];
        const int mr = m - p.m_begin[oseg];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx + 16 * j;
            if (n >= p.N) continue;
            if (p.epilogue == kEpiSwigluBwd) {
                const float g = ld(static_cast<const T*>(p.G) + (long long)m * p.ldgu + n);
                const float u = ld(static_cast<const T*>(p.U) + (long long)m * p.ldgu + n);
                const float d = (float)(T)acc[i][j];
                const float sg = 1.f / (1.f + expf(-g));
                st(C + (long long)m * ldc + n, d * u * sg * (1.f + g * (1.f - sg)));
                st(C + (long long)m * ldc + p.N + n, d * g * sg);
                if (p.act_out) st(static_cast<T*>(p.act_out) + (long long)m * p.N + n, g * sg * u);
            } else {
                T* dst = C + (long long)mr * ldc + n;
                float v = acc[i][j];
                if (p.accumulate) v += ld(dst);
                st(dst, v);
            }
        }
    }
}

int launch_gemm_generic(const GemmDesc& d, hipStream_t stream) {
    GenericGemmParams p;
    p.M = d.M; p.N = d.N; p.n_seg = d.n_seg; p.n_out = d.n_out; p.accumulate = d.accumulate;
    p.a_kmajor = d.a_kmajor; p.b_kmajor = d.b_kmajor;
    for (int s = 0; s < kMaxGemmSegs; ++s) {
        const bool on = s < d.n_seg;
        p.A[s] = on ? d.seg[s].A : nullptr;
        p.B[s] = on ? d.seg[s].B : nullptr;
        p.K[s] = on ? d.seg[s].K : 0;
        p.lda[s] = on ? d.seg[s].lda : 0;
        p.ldb[s] = on ? d.seg[s].ldb : 0;
    }
    for (int s = 0; s < kMaxGemmOuts; ++s) {
        const bool oo = s < d.n_out;
        p.C[s] = oo ? d.out[s].C : nullptr;
        p.m_begin[s] = oo ? d.out[s].m_begin : 0x7fffffff;
        p.ldc[s] = oo ? d.out[s].ldc : 0;
    }
    p.epilogue = d.epilogue; p.G = d.G; p.U = d.U; p.ldgu = d.ldgu; p.act_out = d.act_out;
    p.row_mask = d.row_mask;
    dim3 grid(ceil_div(d.N, 64), ceil_div(d.M, 64));
    if (d.dtype == ALCH_BF16)
        k_gemm_generic<__bf16><<<grid, 256, 0, stream>>>(p);
    else
        k_gemm_generic<float><<<grid, 256, 0, stream>>>(p);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_gemm(const GemmDesc& d, hipStream_t stream) {
    if (d.M <= 0 || d.N <= 0) return ALCH_OK;
    double k_total = 0;
    for (int s = 0; s < d.n_seg; ++s) k_total += d.seg[s].K;
    // a size that lives on the device is not known here: such launches are traced with zero work and the
    // caller accounts for them from the row count it knows
    const bool dev_sized = d.m_dev || d.k_dev;
    const double flops = dev_sized ? 0.0 : 2.0 * d.M * d.N * k_total;
    const size_t E = dtype_size(d.dtype);
    const double bytes = dev_sized ? 0.0 : ((double)d.M * k_total + (double)d.N * k_total + (double)d.M * d.N) * E;
    if (dev_sized && !gemm_mfma_supported(d))
        return fail(ALCH_ERR_UNSUPPORTED, "device-resident sizes need the matrix-core kernel (bf16, aligned, K %% 64 == 0)");
    if (gemm_mfma_supported(d)) {
        TraceScope ts(kTraceGemmMfma, flops, bytes, stream);
        return launch_gemm_mfma(d, stream);
    }
    TraceScope ts(kTraceGemmGeneric, flops, bytes, stream);
    return launch_gemm_generic(d, stream);
}

}  // namespace alch
