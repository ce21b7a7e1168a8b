// bf16 GEMM on the gfx950 matrix cores: C[M,N] (+)= sum_s A_s(M,K_s) B_s(K_s,N), fp32 accumulate.
//
// This one kernel carries all dense contractions of the decoder-layer backward pass
// (Section 4.2 / 4.3.2 of the paper: per-layer backward from saved activations): the
// data gradients (dY.W, activation k-major x weight n-major), the weight gradients
// (dOut^T.Act, both operands token-major, contraction over tokens) and the forward
// projections (x.W^T, both k-major).
//
// Design for CDNA4:
//   * 256x256 tile per work-group, contraction in steps of 32, 4 wavefronts of 64 lanes, each owning 128x128 of the
//     tile as 4x4 MFMA 32x32x16 bf16 accumulators (256 accumulator registers per lane).
//   * Tiles are fetched HBM/L2 -> LDS with 16-byte direct-to-LDS buffer loads (no
//     registers in between) into a ring of stages that fills the 160 KB LDS: five stages of
//     [A 256x32 | B 32x256], or, when A is k-major, three 64-k-wide super-stages of A and four stages
//     of B, so that every load of A covers whole 128-byte lines (see tile_offsets_wide).
//     A direct-to-LDS load writes lane-linearly, so the bank-conflict swizzle is applied
//     by permuting which global 16-byte chunk each lane fetches.
//   * Operands whose contraction index is contiguous in memory are read from LDS with
//     ds_read_b128; operands whose contraction index is the row (token) index are read
//     with the transposing ds_read_b64_tr_b16, so no transposed copy is ever made.
//   * Out-of-range rows/columns (ragged token counts) come back as zeros from the buffer
//     load's range check; stores are predicated.
//   * Work-groups are numbered so that each of the 8 XCDs (one L2 each) works on a
//     compact patch of output tiles.
//   * The grid is persistent, one work-group per compute unit, each walking its share of the tiles
//     round by round.  When the last round would hold tiles for at most half of the compute units, it
//     is left to a second launch (the kSplit instantiation) in which s work-groups of the same XCD
//     share a tile, each taking 1/s of the contraction and leaving an fp32 partial tile in a scratch
//     buffer; k_gemm_split_finish adds the s partials in a fixed order and writes the output
//     (deterministic, no atomics).
#include "kernels.h"

namespace alch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define ALCH_LDS(p) ((__attribute__((address_space(3))) void*)(p))

static constexpr int BM = 256, BN = 256, BK = 32;
static constexpr int kStages = 5;                        // 5 x 32 KB = the whole 160 KB LDS
static constexpr int kOperandStageBytes = 256 * BK * 2;  // 16 KB per operand per stage
static constexpr int kLoadsPerTile = 8;                  // direct-to-LDS instructions per wave per k-tile (A + B)
static constexpr uint32_t kOobOffset = 0x80000000u;      // >= any num_records we set
static constexpr uint32_t kMaxRecords = 0x80000000u;
static constexpr int kGroupM = 4;                        // tile rows per raster band

struct MfmaGemmParams {
    int M, N, n_seg, n_out, accumulate, tiles_m, tiles_n;
    // optional device-resident sizes (row compaction decided on the device): the effective M, or the
    // effective K of every operand pair, is min(*ptr, host value)
    const int* m_dev;
    const int* k_dev;
    const __bf16* A[kMaxGemmSegs];
    const __bf16* B[kMaxGemmSegs];
    int K[kMaxGemmSegs];
    long long lda[kMaxGemmSegs], ldb[kMaxGemmSegs];
    __bf16* C[3];
    int m_begin[3];
    long long ldc[3];
    int epilogue;
    const __bf16* G;
    const __bf16* U;
    long long ldgu;
    __bf16* act_out;
    // Tiles q < q_end of every XCD's share are computed whole by the plain instantiation.  The kSplit
    // instantiation computes the tiles q_end .. of the share, split_s work-groups per tile, partial tiles
    // [tile of the split round][part][256][256] fp32 in split_ws.
    int q_end;
    float* split_ws;
    int split_s, split_per;  // parts per tile; k-tiles per part (counted over all operand pairs in order)
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

// Per-lane byte offsets (relative to the tile origin) of the 4 direct-to-LDS loads a wave
// issues for one operand tile.  LDS slot s (16-byte units) = (wave*4 + j)*64 + lane.
//   k-major tile [256 rows][32 k]: slot = row*4 + (c ^ ((row>>2)&3)), c = 16-byte chunk in the row
//   mn-major tile [32 k][256 cols]: slot = k*32 + (c ^ (4*(k&3)))
template <bool KMAJOR>
__device__ __forceinline__ void tile_offsets(uint32_t (&voff)[4], int wave, int lane, long long ld, int valid) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int s = (wave * 4 + j) * 64 + lane;
        if (KMAJOR) {
            const int row = s >> 2, c = (s & 3) ^ ((row >> 2) & 3);
            voff[j] = row < valid ? (uint32_t)((row * ld + c * 8) * 2) : kOobOffset;
        } else {
            const int k = s >> 5, c = (s & 31) ^ (4 * (k & 3));
            voff[j] = c * 8 < valid ? (uint32_t)((k * ld + c * 8) * 2) : kOobOffset;
        }
    }
}

__device__ __forceinline__ void issue_tile(i32x4 r, uint32_t stage_addr, int wave, const uint32_t (&voff)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) dma16(r, stage_addr + (uint32_t)(wave * 4 + j) * 1024u, voff[j]);
}

// Fragment (8 consecutive-k bf16 per lane for one 32-wide block of rows/cols) from an LDS tile.
template <bool KMAJOR>
__device__ __forceinline__ bf16x8 read_frag(const char* stage, int idx0 /*first row/col of the 32-block*/, int kk, int lane) {
    if (KMAJOR) {
        const int row = idx0 + (lane & 31);
        const int c = (kk * 2 + (lane >> 5)) ^ ((row >> 2) & 3);
        return *reinterpret_cast<const bf16x8*>(stage + row * 64 + c * 16);
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

// ---- k-major A staged 64 k wide ---------------------------------------------------------------
// A k-major tile fetched 32 k at a time takes 64 bytes of every row: each 128-byte line then crosses the
// L2 -> L1 path twice (once per k-tile; the 32 KB L1 has long lost it by the second time).  With AK the A
// operand is therefore staged in super-stages of 64 k: [2 halves of 128 rows][128 bytes], 32 KB, three of
// them, and one wave-wide load covers 8 whole lines.  A super-stage is filled by two batches (rows 0-127,
// rows 128-255), one per k-tile step, so the loads per step stay what they are for the 32-wide layout; the
// B operand keeps 32-wide stages, four of them, behind the three super-stages (96 + 64 = 160 KB).
//   slot (16-byte units) inside a half = rl*8 + (c ^ ((rl>>1)&7)), rl = row & 127, c = 16-byte chunk of the
//   row's 64 k: 16 consecutive rows at one logical chunk then cover all 64 banks once (ds_read_b128).
__device__ __forceinline__ void tile_offsets_wide(uint32_t (&voff)[8], int wave, int lane, long long ld, int valid) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int sl = (wave * 4 + j) * 64 + lane;
            const int rl = sl >> 3, c = (sl & 7) ^ ((rl >> 1) & 7), row = h * 128 + rl;
            voff[h * 4 + j] = row < valid ? (uint32_t)((row * ld + c * 8) * 2) : kOobOffset;
        }
}

// fragment of k-tile `par` (0/1) of a super-stage: rows idx0 + (lane&31), k = par*32 + kk*16 + 8*(lane>>5) ..+7
__device__ __forceinline__ bf16x8 read_frag_wide(const char* sup, int par, int idx0, int kk, int lane) {
    const int row = idx0 + (lane & 31), rl = row & 127;
    const int c = (par * 4 + kk * 2 + (lane >> 5)) ^ ((rl >> 1) & 7);
    return *reinterpret_cast<const bf16x8*>(sup + (row >> 7) * kOperandStageBytes + rl * 128 + c * 16);
}

struct Frags {
    bf16x8 a[4], b[4];
};

template <bool AK, bool BKM>
__device__ __forceinline__ void read_frags(Frags& f, const char* sa, const char* sb, int wm, int wn, int kk, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f.a[i] = read_frag<AK>(sa, wm * 128 + i * 32, kk, lane);
#pragma unroll
    for (int i = 0; i < 4; ++i) f.b[i] = read_frag<BKM>(sb, wn * 128 + i * 32, kk, lane);
}

__device__ __forceinline__ void mfma_block(const Frags& f, f32x16 (&acc)[4][4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}

__device__ __forceinline__ float bf2f(__bf16 v) { return (float)v; }

template <int I> struct IntC { static constexpr int value = I; };
template <typename F> __device__ __forceinline__ void static_for4(F&& f) {
    f(IntC<0>{});
    f(IntC<1>{});
    f(IntC<2>{});
    f(IntC<3>{});
}

template <bool AK, bool BKM, bool kSplit = false>
__global__ __launch_bounds__(256) void k_gemm_mfma(MfmaGemmParams p) {
    // kStages pipeline stages of [A tile 16 KB | B tile 16 KB]
    __shared__ __attribute__((aligned(1024))) char smem[kStages * 2 * kOperandStageBytes];
    const uint32_t lds0 = (uint32_t)(uintptr_t)ALCH_LDS(smem);
    constexpr int kStage = 2 * kOperandStageBytes;
    // AK: A in three 64-wide super-stages, B in four 32-wide stages behind them (see tile_offsets_wide);
    // otherwise kStages stages of [A | B].  kU = steps after which every ring is back at its first stage.
    constexpr bool kWide = AK;
    constexpr int kU = kWide ? 12 : kStages;
    constexpr int kDepth = kWide ? 4 : kStages;  // k-tiles of B (and their share of A) resident at a time
    constexpr uint32_t kWideB0 = 3 * kStage;
    auto a_off = [](int st) -> uint32_t { return kWide ? (uint32_t)((st / 2) % 3) * kStage : (uint32_t)(st % kStages) * kStage; };
    auto b_off = [](int st) -> uint32_t {
        return kWide ? kWideB0 + (uint32_t)(st % 4) * kOperandStageBytes : (uint32_t)(st % kStages) * kStage + kOperandStageBytes;
    };

    // ---- work-group -> output tile: XCD-contiguous chunks, banded raster inside a chunk
    // The grid is persistent (one work-group per compute unit): each work-group walks its share of
    // the tiles, so the stores of one tile drain while the next tile's loads are already in flight.
    const int Mv = p.m_dev ? min(__builtin_amdgcn_readfirstlane(*p.m_dev), p.M) : p.M;
    const int tiles_m = p.m_dev ? (Mv + BM - 1) / BM : p.tiles_m;
    const int nt = tiles_m * p.tiles_n;
    const int per_xcd = (nt + 7) / 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    // kSplit: one tile per work-group; work-group w of an XCD takes part w / rem of tile q_end + w % rem
    const int rem = per_xcd - p.q_end;
    const int ks = kSplit ? (int)(blockIdx.x / 8) / rem : 0;
    // (q_end comes from the host's tile count; with a device-resident row count the XCD's share may be shorter)
    for (int q = kSplit ? p.q_end + (int)(blockIdx.x / 8) % rem : (int)(blockIdx.x / 8); q < (kSplit ? per_xcd : min(p.q_end, per_xcd));
         q += kSplit ? per_xcd : (int)(gridDim.x / 8)) {
    const int t = (blockIdx.x % 8) * per_xcd + q;
    if (t >= nt) break;
    const int band_tiles = kGroupM * p.tiles_n;
    const int band = t / band_tiles, in_band = t % band_tiles;
    const int band_rows = min(kGroupM, tiles_m - band * kGroupM);
    const int tm = band * kGroupM + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    int seg_kt0 = 0;  // kSplit: k-tiles of the operand pairs before this one
    for (int seg = 0; seg < p.n_seg; ++seg) {
        const long long lda = p.lda[seg], ldb = p.ldb[seg];
        const int K = p.k_dev ? min(__builtin_amdgcn_readfirstlane(*p.k_dev), p.K[seg]) : p.K[seg];
        int nk = (K + BK - 1) / BK;
        const char *pa, *pb, *enda, *endb;
        long long stepa, stepb;
        if (AK) {
            pa = (const char*)(p.A[seg] + (long long)m0 * lda);
            enda = (const char*)(p.A[seg] + (long long)(Mv - 1) * lda + K);
            stepa = BK * 2;
        } else {
            pa = (const char*)(p.A[seg] + m0);
            enda = (const char*)(p.A[seg] + (long long)(K - 1) * lda + Mv);
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
        if (kSplit) {  // this work-group's share [ks*per, (ks+1)*per) of the k-tiles of all pairs, cut to this pair
            const int lo = min(max(ks * p.split_per - seg_kt0, 0), nk), hi = min(max((ks + 1) * p.split_per - seg_kt0, 0), nk);
            seg_kt0 += nk;
            if (hi <= lo) continue;
            nk = hi - lo;
            pa += (long long)lo * stepa;
            pb += (long long)lo * stepb;
        }
        uint32_t va[kWide ? 8 : 4], vb[4];
        if constexpr (kWide) tile_offsets_wide(va, wave, lane, lda, Mv - m0);
        else tile_offsets<AK>(va, wave, lane, lda, Mv - m0);
        tile_offsets<BKM>(vb, wave, lane, ldb, p.N - n0);

        // Loads of the next k-tile go out one instruction at a time between MFMAs (a burst of
        // eight would hold the wave at the issue stage while the texture path drains).  Past the
        // last tile the same loads are issued against an empty buffer (they fetch nothing and
        // write zeros nobody reads), so the outstanding-load count is the same in every iteration.
        // The stream state (tile base address, bytes left in the operand) is kept in scalar registers
        // and advanced with scalar instructions, off the vector pipeline that feeds the MFMAs.
        int tiles_left = nk;
        uint32_t a_lo, a_hi, b_lo, b_hi;
        int a_rem, b_rem;
        {
            const uint64_t ua = (uint64_t)pa, ub = (uint64_t)pb;
            const long long la = enda - pa, lb = endb - pb;
            a_lo = __builtin_amdgcn_readfirstlane((uint32_t)ua);
            a_hi = __builtin_amdgcn_readfirstlane((uint32_t)(ua >> 32) & 0xffffu);
            a_rem = __builtin_amdgcn_readfirstlane((int)(la < 0 ? 0 : (la > 0x7fffffffLL ? 0x7fffffffLL : la)));
            b_lo = __builtin_amdgcn_readfirstlane((uint32_t)ub);
            b_hi = __builtin_amdgcn_readfirstlane((uint32_t)(ub >> 32) & 0xffffu);
            b_rem = __builtin_amdgcn_readfirstlane((int)(lb < 0 ? 0 : (lb > 0x7fffffffLL ? 0x7fffffffLL : lb)));
        }
        const int sa_step = __builtin_amdgcn_readfirstlane((int)stepa);
        const int sb_step = __builtin_amdgcn_readfirstlane((int)stepb);
        i32x4 ra, rb;
        auto open_next = [&]() {
            // resources of the next k-tile (an exhausted stream gets an empty buffer), then advance
            int na, nbb;
            asm volatile("s_cmp_gt_i32 %2, 0\n\ts_cselect_b32 %0, %3, 0\n\ts_cselect_b32 %1, %4, 0"
                         : "=&s"(na), "=&s"(nbb)
                         : "s"(tiles_left), "s"(a_rem), "s"(b_rem)
                         : "scc");
            ra[0] = (int)a_lo; ra[1] = (int)a_hi; ra[2] = na; ra[3] = 0x00020000;
            rb[0] = (int)b_lo; rb[1] = (int)b_hi; rb[2] = nbb; rb[3] = 0x00020000;
            asm volatile("s_add_u32 %0, %0, %7\n\ts_addc_u32 %1, %1, 0\n\ts_sub_i32 %2, %2, %7\n\ts_max_i32 %2, %2, 0\n\t"
                         "s_add_u32 %3, %3, %8\n\ts_addc_u32 %4, %4, 0\n\ts_sub_i32 %5, %5, %8\n\ts_max_i32 %5, %5, 0\n\t"
                         "s_sub_i32 %6, %6, 1"
                         : "+s"(a_lo), "+s"(a_hi), "+s"(a_rem), "+s"(b_lo), "+s"(b_hi), "+s"(b_rem), "+s"(tiles_left)
                         : "s"(sa_step), "s"(sb_step)
                         : "scc");
        };
        // kWide: the two streams advance separately.  A moves by 128 bytes (64 k) after every second batch
        // (a_inc alternates 0, 128); its batches are counted in a_left, B's k-tiles in tiles_left.
        int a_left = (nk + 1) & ~1, a_inc = 0;
        auto open_a = [&]() {
            int na;
            asm volatile("s_cmp_gt_i32 %1, 0\n\ts_cselect_b32 %0, %2, 0" : "=&s"(na) : "s"(a_left), "s"(a_rem) : "scc");
            ra[0] = (int)a_lo; ra[1] = (int)a_hi; ra[2] = na; ra[3] = 0x00020000;
            asm volatile("s_add_u32 %0, %0, %4\n\ts_addc_u32 %1, %1, 0\n\ts_sub_i32 %2, %2, %4\n\ts_max_i32 %2, %2, 0\n\t"
                         "s_sub_i32 %4, 128, %4\n\ts_sub_i32 %3, %3, 1"
                         : "+s"(a_lo), "+s"(a_hi), "+s"(a_rem), "+s"(a_left), "+s"(a_inc)
                         :
                         : "scc");
        };
        auto open_b = [&]() {
            int nbb;
            asm volatile("s_cmp_gt_i32 %1, 0\n\ts_cselect_b32 %0, %2, 0" : "=&s"(nbb) : "s"(tiles_left), "s"(b_rem) : "scc");
            rb[0] = (int)b_lo; rb[1] = (int)b_hi; rb[2] = nbb; rb[3] = 0x00020000;
            asm volatile("s_add_u32 %0, %0, %4\n\ts_addc_u32 %1, %1, 0\n\ts_sub_i32 %2, %2, %4\n\ts_max_i32 %2, %2, 0\n\t"
                         "s_sub_i32 %3, %3, 1"
                         : "+s"(b_lo), "+s"(b_hi), "+s"(b_rem), "+s"(tiles_left)
                         : "s"(sb_step)
                         : "scc");
        };
        // Refill issued in step `st`: !kWide: k-tile st + kStages of both operands into the stage of k-tile st.
        // kWide: A batch st + 5 = half (st+5)&1 of super-tile (st+5)/2, B k-tile st + 4 into the stage of k-tile st.
#define ALCH_DMA_A(st, j)                                                                                              \
    dma16(ra, lds0 + (kWide ? a_off((st) + 5) + (uint32_t)(((st) + 5) & 1) * kOperandStageBytes : a_off(st)) +          \
                  (uint32_t)(wave * 4 + (j)) * 1024u, va[kWide ? (((st) + 5) & 1) * 4 + (j) : (j)])
#define ALCH_DMA_B(st, j) dma16(rb, lds0 + b_off(st) + (uint32_t)(wave * 4 + (j)) * 1024u, vb[j])
#define ALCH_MFMA(F, i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F.b[j], F.a[i], acc[i][j], 0, 0, 0)
#define ALCH_SB() __builtin_amdgcn_sched_barrier(0)
        // fragment reads of k-tile step `st`
        auto frag_a = [&](int st, int kk, int i) -> bf16x8 {
            if constexpr (kWide) return read_frag_wide(smem + a_off(st), st & 1, wm * 128 + i * 32, kk, lane);
            else return read_frag<AK>(smem + a_off(st), wm * 128 + i * 32, kk, lane);
        };
#define ALCH_RA(F, st, kk, i) F.a[i] = frag_a(st, kk, i)
#define ALCH_RB(F, st, kk, i) F.b[i] = read_frag<BKM>(smem + b_off(st), wn * 128 + (i) * 32, kk, lane)

        // all waves are done with the previous segment's stages before they are refilled
        __syncthreads();
        if constexpr (kWide) {
            // A batches 0..4 (steps -5..-1 of the refill numbering) and B k-tiles 0..3; k-tile 0 needs the
            // first two batches and B k-tile 0: they go first, the 24 loads behind them may still be in flight
#pragma unroll
            for (int b = 0; b < 5; ++b) {
                open_a();
#pragma unroll
                for (int j = 0; j < 4; ++j) ALCH_DMA_A(b - 5, j);
                if (b >= 1) {
                    open_b();
#pragma unroll
                    for (int j = 0; j < 4; ++j) ALCH_DMA_B(b - 1, j);
                }
            }
            asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        } else {
#pragma unroll
            for (int s = 0; s < kStages; ++s) {
                open_next();
#pragma unroll
                for (int j = 0; j < 4; ++j) { ALCH_DMA_A(s, j); ALCH_DMA_B(s, j); }
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerTile * (kStages - 1)) : "memory");
        }
        __syncthreads();
        Frags f0, f1;
#pragma unroll
        for (int i = 0; i < 4; ++i) { ALCH_RA(f0, 0, 0, i); ALCH_RB(f0, 0, 0, i); }
        for (int kt = 0; kt < nk; kt += kU) {
#pragma unroll
            for (int s = 0; s < kU; ++s) {
                if (kt + s < nk) {
                    const int st = s, stn = (s + 1) % kU;
                    // ---- first half: MFMAs on k 0..15 of this stage, fragment reads for k 16..31
                    ALCH_SB();
                    ALCH_RA(f1, st, 1, 0); ALCH_RA(f1, st, 1, 1); ALCH_MFMA(f0, 0, 0); ALCH_MFMA(f0, 0, 1); ALCH_SB();
                    ALCH_RA(f1, st, 1, 2); ALCH_RA(f1, st, 1, 3); ALCH_MFMA(f0, 0, 2); ALCH_MFMA(f0, 0, 3); ALCH_SB();
                    ALCH_RB(f1, st, 1, 0); ALCH_RB(f1, st, 1, 1); ALCH_MFMA(f0, 1, 0); ALCH_MFMA(f0, 1, 1); ALCH_SB();
                    ALCH_RB(f1, st, 1, 2); ALCH_RB(f1, st, 1, 3); ALCH_MFMA(f0, 1, 2); ALCH_MFMA(f0, 1, 3); ALCH_SB();
                    ALCH_MFMA(f0, 2, 0); ALCH_MFMA(f0, 2, 1); ALCH_MFMA(f0, 2, 2); ALCH_MFMA(f0, 2, 3);
                    ALCH_MFMA(f0, 3, 0); ALCH_MFMA(f0, 3, 1); ALCH_MFMA(f0, 3, 2); ALCH_MFMA(f0, 3, 3);
                    ALCH_SB();
                    // k-tile kt+s+1 has landed (this wave's share), and this wave's reads of stage s are done
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kLoadsPerTile * (kDepth - 2)) : "memory");
                    __syncthreads();
                    // ---- second half: MFMAs on k 16..31, refill of stage s, fragment reads of the next stage
                    if constexpr (kWide) { open_a(); open_b(); }
                    else open_next();
                    ALCH_SB();
                    ALCH_DMA_A(s, 0); ALCH_RA(f0, stn, 0, 0); ALCH_RA(f0, stn, 0, 1); ALCH_MFMA(f1, 0, 0); ALCH_MFMA(f1, 0, 1); ALCH_SB();
                    ALCH_DMA_A(s, 1); ALCH_RA(f0, stn, 0, 2); ALCH_RA(f0, stn, 0, 3); ALCH_MFMA(f1, 0, 2); ALCH_MFMA(f1, 0, 3); ALCH_SB();
                    ALCH_DMA_A(s, 2); ALCH_RB(f0, stn, 0, 0); ALCH_MFMA(f1, 1, 0); ALCH_MFMA(f1, 1, 1); ALCH_SB();
                    ALCH_DMA_A(s, 3); ALCH_RB(f0, stn, 0, 1); ALCH_MFMA(f1, 1, 2); ALCH_MFMA(f1, 1, 3); ALCH_SB();
                    ALCH_DMA_B(s, 0); ALCH_RB(f0, stn, 0, 2); ALCH_MFMA(f1, 2, 0); ALCH_MFMA(f1, 2, 1); ALCH_SB();
                    ALCH_DMA_B(s, 1); ALCH_RB(f0, stn, 0, 3); ALCH_MFMA(f1, 2, 2); ALCH_MFMA(f1, 2, 3); ALCH_SB();
                    ALCH_DMA_B(s, 2); ALCH_MFMA(f1, 3, 0); ALCH_MFMA(f1, 3, 1); ALCH_SB();
                    ALCH_DMA_B(s, 3); ALCH_MFMA(f1, 3, 2); ALCH_MFMA(f1, 3, 3); ALCH_SB();
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef ALCH_DMA_A
#undef ALCH_DMA_B
#undef ALCH_MFMA
#undef ALCH_SB
#undef ALCH_RA
#undef ALCH_RB
    }

    if constexpr (kSplit) {
        // fp32 partial tile, row-major [256][256]: block (i, j) holds (see below) row i*32 + (lane&31) and, in
        // registers 4b..4b+3, columns j*32 + 8b + 4*(lane>>5) + 0..3 of the wave's 128x128 quarter
        float* ws = p.split_ws + ((size_t)(((blockIdx.x % 8) * rem + (q - p.q_end)) * p.split_s + ks)) * (BM * BN) +
                    (wm * 128 + (lane & 31)) * BN + wn * 128 + 4 * (lane >> 5);
        static_for4([&](auto ic) {
            constexpr int i = decltype(ic)::value;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    f32x4 v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = acc[i][j][4 * b + r];
                    *reinterpret_cast<f32x4*>(ws + i * 32 * BN + j * 32 + 8 * b) = v;
                }
        });
    } else {
    // ---- epilogue.  The MFMAs were issued with the operand roles swapped, so block (i, j) holds
    // the transposed 32x32 result: this lane owns output row m = .. + i*32 + (lane&31) and, in
    // registers 4b..4b+3, the four consecutive columns n = .. + j*32 + 8b + 4*(lane>>5) + 0..3.
    int oseg = 0;
#pragma unroll
    for (int s = 1; s < 3; ++s)
        if (s < p.n_out && m0 >= p.m_begin[s]) oseg = s;
    __bf16* __restrict__ C = p.C[oseg];
    const long long ldc = p.ldc[oseg];
    const int mrel0 = m0 - p.m_begin[oseg];
    const int m_end = (oseg + 1 < p.n_out ? min(p.m_begin[oseg + 1], Mv) : Mv);
    const int half = lane >> 5;

    if (!p.accumulate) {
        // Stage the wave's 128x128 bf16 result through the (now idle) pipeline LDS so that it leaves
        // as whole 256-byte row segments: 8-byte LDS writes, 16-byte LDS reads, 16-byte global stores.
        constexpr int kRowStride = 256;  // chunks XOR-ed with the row: 8-byte writes 2-way, 16-byte reads conflict-free
        char* stage = smem + wave * (128 * kRowStride);
        __syncthreads();  // every wave's loads have landed and every wave is done reading the pipeline
        static_for4([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            char* row = stage + (i * 32 + (lane & 31)) * kRowStride;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    bf16x4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = (__bf16)acc[i][j][4 * b + r];
                    *reinterpret_cast<bf16x4*>(row + ((((4 * j + b) ^ (lane & 15)) << 4) | (half << 3))) = o;
                }
        });
        // (a wave reads back only what it wrote itself: no barrier needed in between)
        const int n = n0 + wn * 128 + (lane & 15) * 8;
        if (p.epilogue == kEpiSwigluBwd) {
            // G and U rows (read once, never again: non-temporal loads keep them out of the way of the operand
            // panels in L2) are fetched eight row-steps at a time before any store is issued: the
            // compiler may not move a load above a store it cannot prove disjoint, and one round trip
            // to memory per row-step would leave the epilogue bound by latency.
            constexpr int kBatch = 8;
#pragma unroll 1
            for (int q0 = 0; q0 < 32; q0 += kBatch) {
                bf16x8 g8[kBatch], u8[kBatch];
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int m = m0 + wm * 128 + 4 * (q0 + k) + (lane >> 4);
                    if (m < Mv && n < p.N) {
                        g8[k] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p.G + (long long)m * p.ldgu + n));
                        u8[k] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p.U + (long long)m * p.ldgu + n));
                    }
                }
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int rl = 4 * (q0 + k) + (lane >> 4);
                    const int m = m0 + wm * 128 + rl;
                    const bf16x8 d8 = *reinterpret_cast<const bf16x8*>(stage + rl * kRowStride + (((lane & 15) ^ (rl & 15)) << 4));
                    if (m < Mv && n < p.N) {
                        bf16x8 dg8, du8, a8;
#pragma unroll
                        for (int r = 0; r < 8; ++r) {
                            const float g = bf2f(g8[k][r]), u = bf2f(u8[k][r]), d = bf2f(d8[r]);
                            const float sg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
                            const float silu = g * sg;
                            dg8[r] = (__bf16)(d * u * sg * (1.f + g * (1.f - sg)));
                            du8[r] = (__bf16)(d * silu);
                            a8[r] = (__bf16)(silu * u);
                        }
                        *reinterpret_cast<bf16x8*>(C + (long long)m * ldc + n) = dg8;
                        *reinterpret_cast<bf16x8*>(C + (long long)m * ldc + p.N + n) = du8;
                        if (p.act_out) *reinterpret_cast<bf16x8*>(p.act_out + (long long)m * p.N + n) = a8;
                    }
                }
            }
        } else {
#pragma unroll 8
            for (int qq = 0; qq < 32; ++qq) {
                const int rl = 4 * qq + (lane >> 4);
                const int ml = wm * 128 + rl;
                const bf16x8 d8 = *reinterpret_cast<const bf16x8*>(stage + rl * kRowStride + (((lane & 15) ^ (rl & 15)) << 4));
                if (m0 + ml < m_end && n < p.N) *reinterpret_cast<bf16x8*>(C + (long long)(mrel0 + ml) * ldc + n) = d8;
            }
        }
    } else {
        // accumulate: C = round(acc + C) with the sum in fp32, straight from the accumulators.  The old
        // values of a 32-row block are all fetched before its first store (see the note on loads above).
        static_for4([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const int ml = wm * 128 + i * 32 + (lane & 31);
            __bf16* row = C + (long long)(mrel0 + ml) * ldc;
            const bool row_ok = m0 + ml < m_end;
            bf16x4 old[4][4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int nn = n0 + wn * 128 + j * 32 + 8 * b + 4 * half;
                    if (row_ok && nn < p.N) old[j][b] = *reinterpret_cast<const bf16x4*>(row + nn);
                }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int nn = n0 + wn * 128 + j * 32 + 8 * b + 4 * half;
                    if (row_ok && nn < p.N) {
                        bf16x4 o;
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[i][j][4 * b + r] + bf2f(old[j][b][r]));
                        *reinterpret_cast<bf16x4*>(row + nn) = o;
                    }
                }
        });
    }
    }  // plain epilogue
    }  // tiles of this work-group
}

// Sum of the partial tiles of the split round -> output.  blockIdx.x: tile of that round (same tile numbering as
// the GEMM kernel), blockIdx.y: slab of 16 rows; a thread handles four consecutive columns of four rows.
__global__ __launch_bounds__(256) void k_gemm_split_finish(MfmaGemmParams p, int per_xcd, int nt) {
    const int rem = per_xcd - p.q_end;
    const int t = (blockIdx.x / rem) * per_xcd + p.q_end + blockIdx.x % rem;
    if (t >= nt) return;
    const int band_tiles = kGroupM * p.tiles_n;
    const int band = t / band_tiles, in_band = t % band_tiles;
    const int band_rows = min(kGroupM, p.tiles_m - band * kGroupM);
    const int m0 = (band * kGroupM + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
    int oseg = 0;
#pragma unroll
    for (int s = 1; s < 3; ++s)
        if (s < p.n_out && m0 >= p.m_begin[s]) oseg = s;
    __bf16* __restrict__ C = p.C[oseg];
    const long long ldc = p.ldc[oseg];
    const int mrel0 = m0 - p.m_begin[oseg];
    const int m_end = (oseg + 1 < p.n_out ? min(p.m_begin[oseg + 1], p.M) : p.M);
    const float* ws = p.split_ws + (size_t)blockIdx.x * p.split_s * (BM * BN);
    const int col = 4 * (threadIdx.x & 63), n = n0 + col;
    if (n >= p.N) return;  // (N is a multiple of 8: a thread's four columns are all inside or all outside)
    const int r0 = blockIdx.y * 16 + (threadIdx.x >> 6);
    if (p.epilogue == kEpiSwigluBwd) {
        // the summed product is dAct (rounded to bf16 as the fused epilogue of the unsplit kernel does); with the
        // saved G, U: dG = dAct U s'(G), dU = dAct silu(G), Act = silu(G) U
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + r0 + 4 * i;
            if (m >= p.M) continue;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            for (int k = 0; k < p.split_s; ++k) v += *reinterpret_cast<const f32x4*>(ws + (size_t)k * (BM * BN) + (r0 + 4 * i) * BN + col);
            const bf16x4 g4 = *reinterpret_cast<const bf16x4*>(p.G + (long long)m * p.ldgu + n);
            const bf16x4 u4 = *reinterpret_cast<const bf16x4*>(p.U + (long long)m * p.ldgu + n);
            bf16x4 dg4, du4, a4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float g = bf2f(g4[e]), u = bf2f(u4[e]), dd = bf2f((__bf16)v[e]);
                const float sg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
                const float silu = g * sg;
                dg4[e] = (__bf16)(dd * u * sg * (1.f + g * (1.f - sg)));
                du4[e] = (__bf16)(dd * silu);
                a4[e] = (__bf16)(silu * u);
            }
            *reinterpret_cast<bf16x4*>(C + (long long)m * ldc + n) = dg4;
            *reinterpret_cast<bf16x4*>(C + (long long)m * ldc + p.N + n) = du4;
            if (p.act_out) *reinterpret_cast<bf16x4*>(p.act_out + (long long)m * p.N + n) = a4;
        }
        return;
    }
    f32x4 v[4];
    bf16x4 old[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {  // all loads first
        const int r = r0 + 4 * i;
        v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (m0 + r < m_end) {
            for (int k = 0; k < p.split_s; ++k) v[i] += *reinterpret_cast<const f32x4*>(ws + (size_t)k * (BM * BN) + r * BN + col);
            if (p.accumulate) old[i] = *reinterpret_cast<const bf16x4*>(C + (long long)(mrel0 + r) * ldc + n);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + 4 * i;
        if (m0 + r < m_end) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (__bf16)(p.accumulate ? v[i][e] + bf2f(old[i][e]) : v[i][e]);
            *reinterpret_cast<bf16x4*>(C + (long long)(mrel0 + r) * ldc + n) = o;
        }
    }
}

bool gemm_mfma_supported(const GemmDesc& d) {
    if (d.dtype != ALCH_BF16 || d.M <= 0 || d.N <= 0 || d.n_seg < 1 || d.n_seg > kMaxGemmSegs || d.n_out < 1 || d.n_out > 3)
        return false;
    if (d.row_mask) return false;
    for (int s = 0; s < d.n_seg; ++s) {
        const GemmSeg& g = d.seg[s];
        if (g.K <= 0 || !aligned16(g.A) || !aligned16(g.B) || g.lda % 8 || g.ldb % 8) return false;
        if ((d.a_kmajor || d.b_kmajor) && g.K % 64) return false;  // no k tail on k-major operands
        if (!d.a_kmajor && d.M % 8) return false;
        if (!d.b_kmajor && d.N % 8) return false;
        if (d.N % 8) return false;  // 16-byte output stores
        if (g.lda > (1 << 21) || g.ldb > (1 << 21)) return false;  // tile extent must stay below 2 GiB
        // the kernel tracks the bytes left in an operand in a signed 32-bit scalar
        const long long a_rows = d.a_kmajor ? d.M : g.K, b_rows = d.b_kmajor ? d.N : g.K;
        if (a_rows * g.lda * 2 >= (1LL << 31) || b_rows * g.ldb * 2 >= (1LL << 31)) return false;
    }
    for (int o = 0; o < d.n_out; ++o) {
        if (d.out[o].ldc % 8 || !aligned16(d.out[o].C)) return false;
        if (d.out[o].m_begin % BM) return false;
        if (o == 0 && d.out[o].m_begin != 0) return false;
        if (o > 0 && d.out[o].m_begin <= d.out[o - 1].m_begin) return false;
    }
    if (d.epilogue == kEpiSwigluBwd && (d.n_out != 1 || d.accumulate || d.ldgu % 8 || (d.act_out && !aligned16(d.act_out)) || !aligned16(d.G) || !aligned16(d.U))) return false;
    return true;
}

int launch_gemm_mfma(const GemmDesc& d, hipStream_t stream) {
    MfmaGemmParams p;
    p.M = d.M;
    p.N = d.N;
    p.n_seg = d.n_seg;
    p.n_out = d.n_out;
    p.accumulate = d.accumulate;
    p.m_dev = d.m_dev;
    p.k_dev = d.k_dev;
    p.tiles_m = ceil_div(d.M, BM);
    p.tiles_n = ceil_div(d.N, BN);
    for (int s = 0; s < kMaxGemmSegs; ++s) {
        const bool on = s < d.n_seg;
        p.A[s] = on ? static_cast<const __bf16*>(d.seg[s].A) : nullptr;
        p.B[s] = on ? static_cast<const __bf16*>(d.seg[s].B) : nullptr;
        p.K[s] = on ? d.seg[s].K : 0;
        p.lda[s] = on ? d.seg[s].lda : 0;
        p.ldb[s] = on ? d.seg[s].ldb : 0;
    }
    for (int s = 0; s < kMaxGemmOuts; ++s) {
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
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        ALCH_HIP_TRY(hipGetDevice(&dev));
        ALCH_HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
        n_cu = v > 8 ? v / 8 * 8 : 8;
    }
    const int grid = ceil_div(nt, 8) * 8 < n_cu ? ceil_div(nt, 8) * 8 : n_cu;
    // Split of the last round (see the header): host-known sizes and a contraction long enough that every part
    // still runs the pipeline for a while (the finish kernel carries the SwiGLU-gradient epilogue if there is one).  A product with tiles for at most half of the compute
    // units (a short batch) has no other round: every tile is split.
    const int per_xcd = ceil_div(nt, 8), wgx = n_cu / 8;
    const int full_q = per_xcd / wgx * wgx, rem = per_xcd - full_q;
    p.q_end = per_xcd;
    p.split_ws = nullptr;
    p.split_s = 1;
    p.split_per = 0;
    int nk_total = 0;
    for (int s = 0; s < d.n_seg; ++s) nk_total += ceil_div(d.seg[s].K, BK);
    if (d.split_ws && aligned16(d.split_ws) && !d.m_dev && !d.k_dev && rem > 0 && 2 * rem <= wgx) {
        int s = wgx / rem < 16 ? wgx / rem : 16;
        if (s > nk_total / 16) s = nk_total / 16;
        if (s > 1 && (size_t)8 * rem * s * BM * BN * sizeof(float) <= d.split_ws_bytes) {
            p.q_end = full_q;
            p.split_ws = static_cast<float*>(d.split_ws);
            p.split_s = s;
            p.split_per = ceil_div(nk_total, s);
            if (d.a_kmajor) p.split_per += p.split_per & 1;  // parts start on a 64-k boundary: whole 128-byte lines of A
        }
    }
    const int grid_split = 8 * rem * p.split_s;
    if (d.a_kmajor && d.b_kmajor) {
        if (p.q_end > 0) k_gemm_mfma<true, true><<<grid, 256, 0, stream>>>(p);
        if (p.split_s > 1) k_gemm_mfma<true, true, true><<<grid_split, 256, 0, stream>>>(p);
    } else if (d.a_kmajor && !d.b_kmajor) {
        if (p.q_end > 0) k_gemm_mfma<true, false><<<grid, 256, 0, stream>>>(p);
        if (p.split_s > 1) k_gemm_mfma<true, false, true><<<grid_split, 256, 0, stream>>>(p);
    } else if (!d.a_kmajor && !d.b_kmajor) {
        if (p.q_end > 0) k_gemm_mfma<false, false><<<grid, 256, 0, stream>>>(p);
        if (p.split_s > 1) k_gemm_mfma<false, false, true><<<grid_split, 256, 0, stream>>>(p);
    } else {
        if (p.q_end > 0) k_gemm_mfma<false, true><<<grid, 256, 0, stream>>>(p);
        if (p.split_s > 1) k_gemm_mfma<false, true, true><<<grid_split, 256, 0, stream>>>(p);
    }
    if (p.split_s > 1) k_gemm_split_finish<<<dim3(8 * rem, BM / 16), 256, 0, stream>>>(p, per_xcd, nt);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
