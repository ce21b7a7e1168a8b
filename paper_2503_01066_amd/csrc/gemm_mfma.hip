// bf16 GEMM on the gfx950 matrix cores: C[M,N] (+)= sum_s A_s(M,K_s) B_s(K_s,N), fp32 accumulate.
//
// This one kernel carries all dense contractions of the decoder-layer backward pass
// (Section 4.2 / 4.3.2 of the paper: per-layer backward from saved activations): the
// data gradients (dY.W, activation k-major x weight n-major), the weight gradients
// (dOut^T.Act, both operands token-major, contraction over tokens) and the forward
// projections (x.W^T, both k-major).
//
// Design for CDNA4:
//   * 256x256x64 tile per work-group, 4 wavefronts of 64 lanes, each owning 128x128 of the
//     tile as 4x4 MFMA 32x32x16 bf16 accumulators (256 accumulator registers per lane).
//   * Tiles are fetched HBM/L2 -> LDS with 16-byte direct-to-LDS buffer loads (no
//     registers in between), double buffered: 2 x (32 KB A + 32 KB B) of the 160 KB LDS.
//     A direct-to-LDS load writes lane-linearly, so the bank-conflict swizzle is applied
//     by permuting which global 16-byte chunk each lane fetches.
//   * Operands whose contraction index is contiguous in memory are read from LDS with
//     ds_read_b128; operands whose contraction index is the row (token) index are read
//     with the transposing ds_read_b64_tr_b16, so no transposed copy is ever made.
//   * Out-of-range rows/columns (ragged token counts) come back as zeros from the buffer
//     load's range check; stores are predicated.
//   * Work-groups are numbered so that each of the 8 XCDs (one L2 each) works on a
//     compact patch of output tiles.
#include "kernels.h"

namespace alch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define ALCH_LDS(p) ((__attribute__((address_space(3))) void*)(p))

static constexpr int BM = 256, BN = 256, BK = 64;
static constexpr int kOperandStageBytes = 256 * BK * 2;  // 32 KB
static constexpr uint32_t kOobOffset = 0x80000000u;      // >= any num_records we set
static constexpr uint32_t kMaxRecords = 0x80000000u;
static constexpr int kGroupM = 4;                        // tile rows per raster band

struct MfmaGemmParams {
    int M, N, n_seg, n_out, accumulate, tiles_m, tiles_n;
    const __bf16* A[3];
    const __bf16* B[3];
    int K[3];
    long long lda[3], ldb[3];
    __bf16* C[3];
    int m_begin[3];
    long long ldc[3];
    int epilogue;
    const __bf16* G;
    const __bf16* U;
    long long ldgu;
    __bf16* act_out;
};

typedef __attribute__((ext_vector_type(4))) int i32x4;

// Buffer resource over [p, p + bytes_left): raw (stride 0), 32-bit data format, so that every
// access at or beyond bytes_left reads as zero.  All parts are forced into scalar registers.
__device__ __forceinline__ i32x4 make_rsrc(const void* p, long long bytes_left) {
    const uint32_t n = bytes_left <= 0 ? 0u : (bytes_left > (long long)kMaxRecords ? kMaxRecords : (uint32_t)bytes_left);
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)n);
    r[3] = 0x00020000;
    return r;
}

// 16 bytes per lane from buffer `r` at byte offset `voff` straight into LDS at
// lds_addr + lane*16.  Written as assembly so that the compiler does not order later LDS
// reads of the other pipeline stage behind it; completion is awaited with vmcnt.
__device__ __forceinline__ void dma16(i32x4 r, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(r)
                 : "memory", "m0");
}

// Per-lane byte offsets (relative to the tile origin) of the 8 direct-to-LDS loads a wave
// issues for one operand tile.  LDS slot s (16-byte units) = (wave*8 + j)*64 + lane.
//   k-major tile [256 rows][64 k]: slot = row*8 + (c ^ ((row>>1)&7)), c = 16-byte chunk in the row
//   mn-major tile [64 k][256 cols]: slot = k*32 + (c ^ (4*(k&3)))
template <bool KMAJOR>
__device__ __forceinline__ void tile_offsets(uint32_t (&voff)[8], int wave, int lane, long long ld,
                                             int rows_valid /*k-major: valid rows*/, int cols_valid /*mn-major: valid cols*/) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int s = (wave * 8 + j) * 64 + lane;
        if (KMAJOR) {
            const int row = s >> 3, c = (s & 7) ^ ((row >> 1) & 7);
            voff[j] = row < rows_valid ? (uint32_t)((row * ld + c * 8) * 2) : kOobOffset;
        } else {
            const int k = s >> 5, c = (s & 31) ^ (4 * (k & 3));
            voff[j] = c * 8 < cols_valid ? (uint32_t)((k * ld + c * 8) * 2) : kOobOffset;
        }
    }
}

__device__ __forceinline__ void issue_tile(i32x4 r, uint32_t stage_addr, int wave, const uint32_t (&voff)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) dma16(r, stage_addr + (uint32_t)(wave * 8 + j) * 1024u, voff[j]);
}

// Fragment (8 consecutive-k bf16 per lane for one 32-wide block of rows/cols) from an LDS tile.
template <bool KMAJOR>
__device__ __forceinline__ bf16x8 read_frag(const char* stage, int idx0 /*first row/col of the 32-block*/, int kk, int lane) {
    if (KMAJOR) {
        const int row = idx0 + (lane & 31);
        const int c = (kk * 2 + (lane >> 5)) ^ ((row >> 1) & 7);
        return *reinterpret_cast<const bf16x8*>(stage + row * 128 + c * 16);
    } else {
        const int g = lane >> 4, i = lane & 15;
        const int col = idx0 + (g & 1) * 16 + 4 * (i & 3);
        const int krow = kk * 16 + 8 * (g >> 1) + (i >> 2);  // + 4 for the second half
        const int chunk = col >> 3, sub = (col & 7) * 2;
        const char* p0 = stage + krow * 512 + ((chunk ^ (4 * (krow & 3))) << 4) + sub;
        const char* p1 = p0 + 4 * 512;  // krow + 4 has the same (krow & 3)
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(p0));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(p1));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
}

template <bool AK, bool BKM>
__device__ __forceinline__ void compute_stage(const char* sa, const char* sb, int wm, int wn, int lane, f32x16 (&acc)[4][4]) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 af[4], bfr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = read_frag<AK>(sa, wm * 128 + i * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) bfr[i] = read_frag<BKM>(sb, wn * 128 + i * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
}

__device__ __forceinline__ float bf2f(__bf16 v) { return (float)v; }

template <int I> struct IntC { static constexpr int value = I; };
template <typename F> __device__ __forceinline__ void static_for4(F&& f) {
    f(IntC<0>{});
    f(IntC<1>{});
    f(IntC<2>{});
    f(IntC<3>{});
}

template <bool AK, bool BKM>
__global__ __launch_bounds__(256) void k_gemm_mfma(MfmaGemmParams p) {
    // [A stage 0 | A stage 1 | B stage 0 | B stage 1], 32 KB each: the stage is an immediate offset
    __shared__ __attribute__((aligned(1024))) char smem[4 * kOperandStageBytes];
    const uint32_t lds0 = (uint32_t)(uintptr_t)ALCH_LDS(smem);
    constexpr int kAOff = 0, kBOff = 2 * kOperandStageBytes, kStage = kOperandStageBytes;

    // ---- work-group -> output tile: XCD-contiguous chunks, banded raster inside a chunk
    const int nt = p.tiles_m * p.tiles_n;
    const int per_xcd = (nt + 7) / 8;
    const int t = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (t >= nt) return;
    const int band_tiles = kGroupM * p.tiles_n;
    const int band = t / band_tiles, in_band = t % band_tiles;
    const int band_rows = min(kGroupM, p.tiles_m - band * kGroupM);
    const int tm = band * kGroupM + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    for (int seg = 0; seg < p.n_seg; ++seg) {
        const long long lda = p.lda[seg], ldb = p.ldb[seg];
        const int K = p.K[seg];
        const int nk = (K + BK - 1) / BK;
        const char *pa, *pb, *enda, *endb;
        long long stepa, stepb;
        if (AK) {
            pa = (const char*)(p.A[seg] + (long long)m0 * lda);
            enda = (const char*)(p.A[seg] + (long long)(p.M - 1) * lda + K);
            stepa = BK * 2;
        } else {
            pa = (const char*)(p.A[seg] + m0);
            enda = (const char*)(p.A[seg] + (long long)(K - 1) * lda + p.M);
            stepa = (long long)BK * lda * 2;
        }
        if (BKM) {
            pb = (const char*)(p.B[seg] + (long long)n0 * ldb);
            endb = (const char*)(p.B[seg] + (long long)(p.N - 1) * ldb + K);
            stepb = BK * 2;
        } else {
            pb = (const char*)(p.B[seg] + n0);
            endb = (const char*)(p.B[seg] + (long long)(K - 1) * ldb + p.N);
            stepb = (long long)BK * ldb * 2;
        }
        uint32_t va[8], vb[8];
        tile_offsets<AK>(va, wave, lane, lda, p.M - m0, p.M - m0);
        tile_offsets<BKM>(vb, wave, lane, ldb, p.N - n0, p.N - n0);

        // all waves are done reading the previous segment's last stage before it is refilled
        __syncthreads();
        issue_tile(make_rsrc(pa, enda - pa), lds0 + kAOff, wave, va);
        issue_tile(make_rsrc(pb, endb - pb), lds0 + kBOff, wave, vb);
        for (int kt = 0; kt < nk; kt += 2) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (kt + 1 < nk) {
                pa += stepa;
                pb += stepb;
                issue_tile(make_rsrc(pa, enda - pa), lds0 + kAOff + kStage, wave, va);
                issue_tile(make_rsrc(pb, endb - pb), lds0 + kBOff + kStage, wave, vb);
            }
            compute_stage<AK, BKM>(smem + kAOff, smem + kBOff, wm, wn, lane, acc);
            if (kt + 1 >= nk) break;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (kt + 2 < nk) {
                pa += stepa;
                pb += stepb;
                issue_tile(make_rsrc(pa, enda - pa), lds0 + kAOff, wave, va);
                issue_tile(make_rsrc(pb, endb - pb), lds0 + kBOff, wave, vb);
            }
            compute_stage<AK, BKM>(smem + kAOff + kStage, smem + kBOff + kStage, wm, wn, lane, acc);
        }
    }

    // ---- epilogue: lane holds column n = n0 + wn*128 + j*32 + (lane&31), rows 8b + 4(lane>>5) + r
    int oseg = 0;
#pragma unroll
    for (int s = 1; s < 3; ++s)
        if (s < p.n_out && m0 >= p.m_begin[s]) oseg = s;
    __bf16* __restrict__ C = p.C[oseg];
    const long long ldc = p.ldc[oseg];
    const int mrel0 = m0 - p.m_begin[oseg];
    const int m_end = (oseg + 1 < p.n_out ? p.m_begin[oseg + 1] : p.M);

    // (the row-block loop is expanded through a template so that every accumulator index is a
    // compile-time constant and the accumulators stay in registers)
    if (p.epilogue == kEpiSwigluBwd) {
        static_for4([&](auto ic) {
            constexpr int i = decltype(ic)::value;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + wn * 128 + j * 32 + (lane & 31);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    if (m < p.M && n < p.N) {
                        const float g = bf2f(p.G[(long long)m * p.ldgu + n]);
                        const float u = bf2f(p.U[(long long)m * p.ldgu + n]);
                        const float d = bf2f((__bf16)acc[i][j][e]);  // dAct is a bf16 tensor of the method
                        const float sg = 1.f / (1.f + __expf(-g));
                        const float silu = g * sg;
                        C[(long long)m * ldc + n] = (__bf16)(d * u * sg * (1.f + g * (1.f - sg)));
                        C[(long long)m * ldc + p.N + n] = (__bf16)(d * silu);
                        if (p.act_out) p.act_out[(long long)m * p.N + n] = (__bf16)(silu * u);
                    }
                }
            }
        });
        return;
    }

    static_for4([&](auto ic) {
        constexpr int i = decltype(ic)::value;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn * 128 + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int ml = wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m0 + ml < m_end && n < p.N) {
                    __bf16* dst = C + (long long)(mrel0 + ml) * ldc + n;
                    float v = acc[i][j][e];
                    if (p.accumulate) v += bf2f(*dst);
                    *dst = (__bf16)v;
                }
            }
        }
    });
}

bool gemm_mfma_supported(const GemmDesc& d) {
    if (d.dtype != ALCH_BF16 || d.M <= 0 || d.N <= 0 || d.n_seg < 1 || d.n_seg > 3 || d.n_out < 1 || d.n_out > 3)
        return false;
    if (d.row_mask) return false;
    for (int s = 0; s < d.n_seg; ++s) {
        const GemmSeg& g = d.seg[s];
        if (g.K <= 0 || !aligned16(g.A) || !aligned16(g.B) || g.lda % 8 || g.ldb % 8) return false;
        if ((d.a_kmajor || d.b_kmajor) && g.K % BK) return false;  // no k tail on k-major operands
        if (!d.a_kmajor && d.M % 8) return false;
        if (!d.b_kmajor && d.N % 8) return false;
        if (g.lda > (1 << 21) || g.ldb > (1 << 21)) return false;  // tile extent must stay below 2 GiB
    }
    for (int o = 0; o < d.n_out; ++o) {
        if (d.out[o].m_begin % BM) return false;
        if (o == 0 && d.out[o].m_begin != 0) return false;
        if (o > 0 && d.out[o].m_begin <= d.out[o - 1].m_begin) return false;
    }
    if (d.epilogue == kEpiSwigluBwd && (d.n_out != 1 || d.accumulate)) return false;
    return true;
}

int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream) {
    MfmaGemmParams p;
    p.M = d.M;
    p.N = d.N;
    p.n_seg = d.n_seg;
    p.n_out = d.n_out;
    p.accumulate = d.accumulate;
    p.tiles_m = ceil_div(d.M, BM);
    p.tiles_n = ceil_div(d.N, BN);
    for (int s = 0; s < 3; ++s) {
        const bool on = s < d.n_seg;
        p.A[s] = on ? static_cast<const __bf16*>(d.seg[s].A) : nullptr;
        p.B[s] = on ? static_cast<const __bf16*>(d.seg[s].B) : nullptr;
        p.K[s] = on ? d.seg[s].K : 0;
        p.lda[s] = on ? d.seg[s].lda : 0;
        p.ldb[s] = on ? d.seg[s].ldb : 0;
        const bool oo = s < d.n_out;
        p.C[s] = oo ? static_cast<__bf16*>(d.out[s].C) : nullptr;
        p.m_begin[s] = oo ? d.out[s].m_begin : 0x7fffffff;
        p.ldc[s] = oo ? d.out[s].ldc : 0;
    }
    p.epilogue = d.epilogue;
    p.G = static_cast<const __bf16*>(d.G);
    p.U = static_cast<const __bf16*>(d.U);
    p.ldgu = d.ldgu;
    p.act_out = static_cast<__bf16*>(d.act_out);
    const int nt = p.tiles_m * p.tiles_n;
    const int grid = ceil_div(nt, 8) * 8;
    if (d.a_kmajor && d.b_kmajor)
        k_gemm_mfma<true, true><<<grid, 256, 0, stream>>>(p);
    else if (d.a_kmajor && !d.b_kmajor)
        k_gemm_mfma<true, false><<<grid, 256, 0, stream>>>(p);
    else if (!d.a_kmajor && !d.b_kmajor)
        k_gemm_mfma<false, false><<<grid, 256, 0, stream>>>(p);
    else
        k_gemm_mfma<false, true><<<grid, 256, 0, stream>>>(p);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
