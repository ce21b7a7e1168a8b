// Causal grouped-query attention, plain version: one wavefront per (token, head) row, fp32
// arithmetic, any head_dim up to 256, float or bf16 storage.  It serves the fp32 storage type
// and head sizes the matrix-core kernels do not take; correctness first.
//
// Backward from the saved record (Section 4.1 of the paper: Q, K, V of the prompt tokens are what
// the serving side keeps): p_ij = exp(q_i.k_j/sqrt(D) - LSE_i) for j <= i in the same sequence,
// dV_j = sum_i p_ij dO_i, ds_ij = p_ij (dO_i.v_j - delta_i), dQ_i = sum_j ds_ij k_j / sqrt(D),
// dK_j = sum_i ds_ij q_i / sqrt(D); K/V gradients are summed over the query heads of a group.
// A sequence with a prefix (responses on the saved KV cache of their prompt, Section 4.1) also sees
// every key of the prefix sequence; the keys of a prefix collect gradient from all sequences that
// name it.
#include "kernels.h"

namespace alch {

template <typename T> __device__ __forceinline__ float ldf(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v) { *p = (T)v; }

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ int find_seq(const int* __restrict__ cu, int n_seqs, int t) {
    int lo = 0, hi = n_seqs;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

static constexpr int kMaxPerLane = 4;  // head_dim <= 256

template <typename T>
__global__ __launch_bounds__(256) void k_attn_fwd_generic(const T* __restrict__ Q, const T* __restrict__ K,
                                                          const T* __restrict__ V, T* __restrict__ O,
                                                          float* __restrict__ LSE, int Ttok, int n_seqs,
                                                          const int* __restrict__ cu, const int* __restrict__ prefix,
                                                          int row_begin, int Hq, int Hkv, int D) {
    const long long row = (long long)row_begin * Hq + (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long long)Ttok * Hq) return;
    const int lane = threadIdx.x & 63;
    const int t = (int)(row / Hq), h = (int)(row % Hq), kv = h / (Hq / Hkv);
    const int seq = find_seq(cu, n_seqs, t);
    const int start = cu[seq];
    const int pre = prefix ? prefix[seq] : -1;
    const int pre_start = pre >= 0 ? cu[pre] : 0, pre_len = pre >= 0 ? cu[pre + 1] - pre_start : 0;
    const float scale = rsqrtf((float)D);
    float q[kMaxPerLane], o[kMaxPerLane];
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        q[e] = d < D ? ldf(Q + ((long long)t * Hq + h) * D + d) : 0.f;
        o[e] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    for (int jj = 0; jj < pre_len + t - start + 1; ++jj) {
        const int j = jj < pre_len ? pre_start + jj : start + jj - pre_len;
        const T* kr = K + ((long long)j * Hkv + kv) * D;
        const T* vr = V + ((long long)j * Hkv + kv) * D;
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < kMaxPerLane; ++e) {
            const int d = lane + 64 * e;
            if (d < D) s += q[e] * ldf(kr + d);
        }
        s = wsum(s) * scale;
        const float mn = fmaxf(m, s);
        const float corr = expf(m - mn), p = expf(s - mn);
        l = l * corr + p;
#pragma unroll
        for (int e = 0; e < kMaxPerLane; ++e) {
            const int d = lane + 64 * e;
            if (d < D) o[e] = o[e] * corr + p * ldf(vr + d);
        }
        m = mn;
    }
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        if (d < D) stf(O + ((long long)t * Hq + h) * D + d, o[e] / l);
    }
    if (lane == 0) LSE[row] = m + logf(l);
}

template <typename T>
__global__ __launch_bounds__(256) void k_attn_bwd_dq_generic(const T* __restrict__ Q, const T* __restrict__ K,
                                                             const T* __restrict__ V, const T* __restrict__ dO,
                                                             const float* __restrict__ LSE,
                                                             const float* __restrict__ delta, T* __restrict__ dQ,
                                                             long long ld, int Ttok, int n_seqs,
                                                             const int* __restrict__ cu, const int* __restrict__ prefix,
                                                             int Hq, int Hkv, int D) {
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long long)Ttok * Hq) return;
    const int lane = threadIdx.x & 63;
    const int t = (int)(row / Hq), h = (int)(row % Hq), kv = h / (Hq / Hkv);
    const int seq = find_seq(cu, n_seqs, t);
    const int start = cu[seq];
    const int pre = prefix ? prefix[seq] : -1;
    const int pre_start = pre >= 0 ? cu[pre] : 0, pre_len = pre >= 0 ? cu[pre + 1] - pre_start : 0;
    const float scale = rsqrtf((float)D);
    float q[kMaxPerLane], go[kMaxPerLane], dq[kMaxPerLane];
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        q[e] = d < D ? ldf(Q + ((long long)t * Hq + h) * D + d) : 0.f;
        go[e] = d < D ? ldf(dO + ((long long)t * Hq + h) * D + d) : 0.f;
        dq[e] = 0.f;
    }
    const float lse = LSE[row], dl = delta[row];
    for (int jj = 0; jj < pre_len + t - start + 1; ++jj) {
        const int j = jj < pre_len ? pre_start + jj : start + jj - pre_len;
        const T* kr = K + ((long long)j * Hkv + kv) * D;
        const T* vr = V + ((long long)j * Hkv + kv) * D;
        float s = 0.f, dp = 0.f, kk[kMaxPerLane];
#pragma unroll
        for (int e = 0; e < kMaxPerLane; ++e) {
            const int d = lane + 64 * e;
            kk[e] = d < D ? ldf(kr + d) : 0.f;
            s += q[e] * kk[e];
            if (d < D) dp += go[e] * ldf(vr + d);
        }
        s = wsum(s) * scale;
        dp = wsum(dp);
        const float ds = expf(s - lse) * (dp - dl);
#pragma unroll
        for (int e = 0; e < kMaxPerLane; ++e) dq[e] += ds * kk[e];
    }
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        if (d < D) stf(dQ + (long long)t * ld + (long long)h * D + d, dq[e] * scale);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_attn_bwd_dkv_generic(const T* __restrict__ Q, const T* __restrict__ K,
                                                              const T* __restrict__ V, const T* __restrict__ dO,
                                                              const float* __restrict__ LSE,
                                                              const float* __restrict__ delta, T* __restrict__ dK,
                                                              T* __restrict__ dV, long long ld, int Ttok,
                                                              int n_seqs, const int* __restrict__ cu,
                                                              const int* __restrict__ prefix, int Hq, int Hkv, int D) {
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long long)Ttok * Hkv) return;
    const int lane = threadIdx.x & 63;
    const int t = (int)(row / Hkv), kv = (int)(row % Hkv), G = Hq / Hkv;
    const int seq = find_seq(cu, n_seqs, t);
    const int end = cu[seq + 1];
    const float scale = rsqrtf((float)D);
    float k[kMaxPerLane], v[kMaxPerLane], dk[kMaxPerLane], dv[kMaxPerLane];
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        k[e] = d < D ? ldf(K + ((long long)t * Hkv + kv) * D + d) : 0.f;
        v[e] = d < D ? ldf(V + ((long long)t * Hkv + kv) * D + d) : 0.f;
        dk[e] = dv[e] = 0.f;
    }
    // query rows: the rest of the key's own sequence, then all rows of every sequence that names it as prefix
    for (int c = seq; c < n_seqs; ++c) {
        if (c > seq && !(prefix && prefix[c] == seq)) continue;
        const int i_first = c == seq ? t : cu[c], i_end = c == seq ? end : cu[c + 1];
        for (int h = kv * G; h < (kv + 1) * G; ++h)
        for (int i = i_first; i < i_end; ++i) {
            const T* qr = Q + ((long long)i * Hq + h) * D;
            const T* gr = dO + ((long long)i * Hq + h) * D;
            float s = 0.f, dp = 0.f, qq[kMaxPerLane], gg[kMaxPerLane];
#pragma unroll
            for (int e = 0; e < kMaxPerLane; ++e) {
                const int d = lane + 64 * e;
                qq[e] = d < D ? ldf(qr + d) : 0.f;
                gg[e] = d < D ? ldf(gr + d) : 0.f;
                s += qq[e] * k[e];
                dp += gg[e] * v[e];
            }
            s = wsum(s) * scale;
            dp = wsum(dp);
            const float p = expf(s - LSE[(long long)i * Hq + h]);
            const float ds = p * (dp - delta[(long long)i * Hq + h]);
#pragma unroll
            for (int e = 0; e < kMaxPerLane; ++e) {
                dv[e] += p * gg[e];
                dk[e] += ds * qq[e];
            }
        }
        if (!prefix) break;
    }
#pragma unroll
    for (int e = 0; e < kMaxPerLane; ++e) {
        const int d = lane + 64 * e;
        if (d < D) {
            stf(dK + (long long)t * ld + (long long)kv * D + d, dk[e] * scale);
            stf(dV + (long long)t * ld + (long long)kv * D + d, dv[e]);
        }
    }
}

template <typename T>
static int attn_bwd_generic_t(const AttnArgs& a, hipStream_t stream) {
    const long long nq = (long long)a.T * a.Hq, nk = (long long)a.T * a.Hkv;
    k_attn_bwd_dq_generic<T><<<(int)((nq + 3) / 4), 256, 0, stream>>>(
        (const T*)a.Q, (const T*)a.K, (const T*)a.V, (const T*)a.dO, a.LSE, a.delta, (T*)a.dQ, a.ld_dqkv, a.T,
        a.n_seqs, a.cu_seqlens, a.prefix, a.Hq, a.Hkv, a.D);
    k_attn_bwd_dkv_generic<T><<<(int)((nk + 3) / 4), 256, 0, stream>>>(
        (const T*)a.Q, (const T*)a.K, (const T*)a.V, (const T*)a.dO, a.LSE, a.delta, (T*)a.dK, (T*)a.dV, a.ld_dqkv,
        a.T, a.n_seqs, a.cu_seqlens, a.prefix, a.Hq, a.Hkv, a.D);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_attn_bwd_generic(const AttnArgs& a, hipStream_t stream) {
    if (a.T <= 0) return ALCH_OK;
    if (a.D > 64 * kMaxPerLane) return fail(ALCH_ERR_UNSUPPORTED, "head_dim %d > %d", a.D, 64 * kMaxPerLane);
    return a.dtype == ALCH_BF16 ? attn_bwd_generic_t<__bf16>(a, stream) : attn_bwd_generic_t<float>(a, stream);
}

int launch_attn_fwd_generic(alch_dtype dt, const void* Q, const void* K, const void* V, void* O, float* LSE, int T,
                            int n_seqs, const int* cu_seqlens, const int* cu_seqlens_host, const int* prefix,
                            int seq_begin, int Hq, int Hkv, int D, hipStream_t stream) {
    const int row_begin = cu_seqlens_host[seq_begin];
    if (T - row_begin <= 0) return ALCH_OK;
    if (D > 64 * kMaxPerLane) return fail(ALCH_ERR_UNSUPPORTED, "head_dim %d > %d", D, 64 * kMaxPerLane);
    const long long nq = (long long)(T - row_begin) * Hq;
    const int grid = (int)((nq + 3) / 4);
    if (dt == ALCH_BF16)
        k_attn_fwd_generic<__bf16><<<grid, 256, 0, stream>>>((const __bf16*)Q, (const __bf16*)K, (const __bf16*)V,
                                                             (__bf16*)O, LSE, T, n_seqs, cu_seqlens, prefix, row_begin, Hq, Hkv, D);
    else
        k_attn_fwd_generic<float><<<grid, 256, 0, stream>>>((const float*)Q, (const float*)K, (const float*)V,
                                                            (float*)O, LSE, T, n_seqs, cu_seqlens, prefix, row_begin, Hq, Hkv, D);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
