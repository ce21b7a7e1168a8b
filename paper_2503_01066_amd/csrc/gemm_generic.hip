// Plain tiled GEMM in fp32 arithmetic for the fp32 storage type and for bf16 problems whose
// shapes or alignments the matrix-core kernel does not take.  Same contract as the
// matrix-core kernel (segments, split outputs, accumulate); correctness first.
#include <algorithm>
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

// The matrix-core kernel addresses an operand through one buffer descriptor and refuses operands of 2 GiB or more.
// The operands that grow with the batch are indexed by tokens: the rows of a k-major A (data gradients, forward)
// or the contraction index of a weight gradient.  A product refused for that reason alone is cut along that
// index into bands the kernel takes: row bands are independent products; contraction bands accumulate into the
// output one after the other (sum in fp32 inside a band, one rounding to the storage type per band).
// Returns true when the product was launched that way (rc holds the status).
static bool launch_gemm_in_bands(const GemmDesc& d, hipStream_t stream, int& rc) {
    if (d.dtype != ALCH_BF16 || d.m_dev || d.k_dev || d.row_mask || d.n_out != 1 || d.out[0].m_begin != 0) return false;
    const long long kLimit = (1LL << 31) - 1;
    const bool rows = d.a_kmajor;                        // bands over M
    const bool contr = !d.a_kmajor && !d.b_kmajor;       // bands over K (single operand pair)
    if (!rows && !contr) return false;
    if (contr && d.n_seg != 1) return false;
    long long ld_max = 1;
    for (int s = 0; s < d.n_seg; ++s) ld_max = std::max(ld_max, contr ? std::max(d.seg[s].lda, d.seg[s].ldb) : d.seg[s].lda);
    if (d.epilogue == kEpiSwigluBwd) ld_max = std::max(ld_max, std::max(d.ldgu, d.out[0].ldc));
    const long long total = rows ? d.M : d.seg[0].K;
    long long band = kLimit / (ld_max * 2) / 256 * 256;
    if (band < 256 || band >= total) return false;       // nothing to gain, or not the reason of the refusal
    auto band_desc = [&](long long b0, long long n) {
        GemmDesc e = d;
        if (rows) {
            e.M = (int)n;
            for (int s = 0; s < d.n_seg; ++s) e.seg[s].A = static_cast<const char*>(d.seg[s].A) + b0 * d.seg[s].lda * 2;
            e.out[0].C = static_cast<char*>(d.out[0].C) + b0 * d.out[0].ldc * 2;
            if (d.epilogue == kEpiSwigluBwd) {
                e.G = static_cast<const char*>(d.G) + b0 * d.ldgu * 2;
                e.U = static_cast<const char*>(d.U) + b0 * d.ldgu * 2;
                if (d.act_out) e.act_out = static_cast<char*>(d.act_out) + b0 * (long long)d.N * 2;
            }
        } else {
            e.seg[0].K = (int)n;
            e.seg[0].A = static_cast<const char*>(d.seg[0].A) + b0 * d.seg[0].lda * 2;
            e.seg[0].B = static_cast<const char*>(d.seg[0].B) + b0 * d.seg[0].ldb * 2;
            e.accumulate = b0 == 0 ? d.accumulate : 1;
        }
        return e;
    };
    for (long long b0 = 0; b0 < total; b0 += band)
        if (!gemm_mfma_supported(band_desc(b0, std::min(band, total - b0)))) return false;
    rc = ALCH_OK;
    for (long long b0 = 0; b0 < total && rc == ALCH_OK; b0 += band) {
        const GemmDesc e = band_desc(b0, std::min(band, total - b0));
        double k_total = 0;
        for (int s = 0; s < e.n_seg; ++s) k_total += e.seg[s].K;
        TraceScope ts(kTraceGemmMfma, 2.0 * e.M * e.N * k_total, ((double)e.M * k_total + (double)e.N * k_total + (double)e.M * e.N) * 2, stream);
        rc = launch_gemm_mfma(e, stream);
    }
    return true;
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
    int rc = ALCH_OK;
    if (launch_gemm_in_bands(d, stream, rc)) return rc;
    TraceScope ts(kTraceGemmGeneric, flops, bytes, stream);
    return launch_gemm_generic(d, stream);
}

}  // namespace alch
