// Causal grouped-query attention on the gfx950 matrix cores, head_dim 128, bf16.
//
// Backward from the saved record (Section 4.1 of the paper: the prompt's Q, K, V stay on the
// GPU after prefill; Section 4.2: the layer's backward consumes them).  Probabilities are
// rebuilt from saved Q, K and LSE, never stored: p_ij = exp(q_i.k_j/sqrt(D) - LSE_i), j <= i.
//
// Two kernels, no atomics, deterministic:
//   dK/dV kernel: a work-group owns 128 keys of one (sequence, kv head) -- 32 per wavefront,
//     their K and V fragments held in registers -- and streams 64-query tiles of Q and dO of
//     every query head of the group through LDS (direct-to-LDS loads, four stages, software pipelined).
//       S = Q K^T, dP = dO V^T            (tile rows from LDS with ds_read_b128)
//       P, dS in the accumulator layout feed straight back as the left operand of
//       dV += P^T dO, dK += dS^T Q        (dO, Q rows read with the transposing LDS read)
//   dQ kernel: a work-group owns 128 queries of one (sequence, query head) and streams 64-key
//     tiles of K and V:  S^T = K Q^T, dP^T = V dO^T, dQ += dS K.
// The LDS tile is [rows][128] bf16 with the 16-byte chunk index XOR-ed by a function of the row
// that makes both the row-major and the transposing reads bank-conflict free.
#include <type_traits>
#include "kernels.h"

namespace alch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

#define ALCH_LDS(p) ((__attribute__((address_space(3))) void*)(p))

static constexpr int kD = 128;
static constexpr int kTileRows = 64;                       // rows of a streamed tile
static constexpr int kTileBytes = kTileRows * kD * 2;      // 16 KB
static constexpr int kStageBytes = 2 * kTileBytes + 1024;  // two tiles + two 64-float vectors (padded)
static constexpr float kLog2e = 1.4426950408889634f;

struct AttnMfmaParams {
    const __bf16 *Q, *K, *V, *O, *dO;
    const float* LSE;
    float* delta;  // written by the dQ kernel (row sums of dO*O), read by the dK/dV kernel
    float* lse2;   // LSE * log2(e), written by the dQ kernel for the dK/dV kernel (its exponent is one fused multiply-add)
    __bf16 *dQ, *dK, *dV;
    const int* cu;
    const int* prefix;     // null, or per sequence: -1 / the earlier sequence whose keys it also attends to
    int n_seqs;
    const int* positions;  // RoPE positions per token, or null: index inside the sequence
    int Hq, Hkv;
    long long ldq, ldk, ldo;  // row strides (elements) of Q/dO, K/V, and of the outputs
    float scale;
    float rope_log2_base;  // > 0: rotate dQ, dK by minus the RoPE angle before they are stored
};

// RoPE backward on one accumulator set: block nb (< 2) holds element d = nb*32 + (lane&31) of a head,
// block nb + 2 its partner d + 64; x'[d] = x[d] cos a + x[d+64] sin a, x'[d+64] = x[d+64] cos a - x[d] sin a
// with a = pos * base^(-2d/128).
__device__ __forceinline__ void rope_backward_rows(f32x16 (&x)[4], const AttnMfmaParams& p, int seq_start, int row0,
                                                  int len, int lane) {
    const int half = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float theta = __builtin_amdgcn_exp2f(-(float)(nb * 32 + (lane & 31)) * (2.0f / kD) * p.rope_log2_base);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = row0 + 8 * (e >> 2) + 4 * half + (e & 3);
            const int pos = (p.positions && r < len) ? p.positions[seq_start + r] : r;
            float sn, cs;
            __sincosf((float)pos * theta, &sn, &cs);
            const float a = x[nb][e], b = x[nb + 2][e];
            x[nb][e] = a * cs + b * sn;
            x[nb + 2][e] = b * cs - a * sn;
        }
    }
}

__device__ __forceinline__ i32x4 rsrc_of(const void* p, long long bytes) {
    const uint32_t n = bytes <= 0 ? 0u : (bytes > 0x7fffffffLL ? 0x7fffffffu : (uint32_t)bytes);
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)n);
    r[3] = 0x00020000;
    return r;
}
__device__ __forceinline__ void dma16(i32x4 r, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(r)
                 : "memory", "m0");
}
__device__ __forceinline__ void dma4(i32x4 r, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(r)
                 : "memory", "m0");
}

// chunk swizzle of the [rows][128] tile: 16 chunks of 16 bytes per row
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// Per-lane byte offsets of one wave's share (4 of 16 loads) of a 64-row tile of rows `ld` elements apart.
__device__ __forceinline__ void tile_voffsets(uint32_t (&voff)[4], long long ld, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int slot = (wave * 4 + j) * 64 + lane;
        const int row = slot >> 4, c = (slot & 15) ^ swz(row);
        voff[j] = (uint32_t)((row * ld + c * 8) * 2);
    }
}
// The loads themselves: tile rows start at `base`, `rows_valid` rows exist (the rest read as zero).
__device__ __forceinline__ void issue_rows_tile(const __bf16* base, long long ld, int rows_valid, uint32_t lds_addr,
                                                int wave, const uint32_t (&voff)[4]) {
    const i32x4 r = rsrc_of(base, rows_valid > 0 ? ((long long)(rows_valid - 1) * ld + kD) * 2 : 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) dma16(r, lds_addr + (uint32_t)(wave * 4 + j) * 1024u, voff[j]);
}
// 64 floats with stride `stride` elements (one per tile row) -> LDS, by one wave
__device__ __forceinline__ void issue_row_scalars(const float* base, long long stride, int rows_valid, uint32_t lds_addr,
                                                  int lane) {
    const i32x4 r = rsrc_of(base, rows_valid > 0 ? ((long long)(rows_valid - 1) * stride + 1) * 4 : 0);
    dma4(r, lds_addr, (uint32_t)(lane * stride * 4));
}

// LDS read addresses.  Every fragment address of a [rows][128] tile is a per-lane constant combined
// with compile-time terms, so the lane parts are computed once per kernel:
//   d-fragments (k = d):   byte = row0*256 + (lane_d ^ (kk << 5)),       lane_d from frag_d_lane()
//   row-fragments (k = row): byte = (row0 + 16*ks)*256 + (lane_r ^ (nb << 6)), lane_r from frag_rows_lane()
// where row0 is a multiple of 32 (XOR and ADD commute with it).
__device__ __forceinline__ uint32_t frag_d_lane(int lane) {
    const int row = lane & 31;
    return (uint32_t)(row * 256 + (((lane >> 5) ^ swz(row)) << 4));
}
// second = 0: tile rows 4*(g>>1) + (i>>2); second = 1: eight rows further down
__device__ __forceinline__ uint32_t frag_rows_lane(int lane, int second) {
    const int g = lane >> 4, i = lane & 15;
    const int col = (g & 1) * 16 + 4 * (i & 3);
    const int r = 4 * (g >> 1) + (i >> 2) + 8 * second;
    return (uint32_t)(r * 256 + (((col >> 3) ^ swz(r)) << 4) + (col & 7) * 2);
}
__device__ __forceinline__ bf16x8 lds_frag_d(const char* tile, uint32_t lane_d, int kk) {
    return *reinterpret_cast<const bf16x8*>(tile + (lane_d ^ (uint32_t)(kk << 5)));
}
__device__ __forceinline__ bf16x8 lds_frag_rows(const char* tile, uint32_t lane_r0, uint32_t lane_r1, int ks, int nb) {
    const char* t = tile + ks * 16 * 256;
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(t + (lane_r0 ^ (uint32_t)(nb << 6))));
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(t + (lane_r1 ^ (uint32_t)(nb << 6))));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int ks) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[8 * ks + e];
    return o;
}

// 16-byte global load of an operand fragment held in registers for the whole kernel:
// rows row0 + (lane&31) of a [rows, ld] matrix (column offset already in base), zero beyond rows_valid
__device__ __forceinline__ bf16x8 global_frag_d(const __bf16* base, long long ld, int row0, int rows_valid, int kk, int lane) {
    const int row = row0 + (lane & 31);
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
    if (row >= rows_valid) return z;
    return *reinterpret_cast<const bf16x8*>(base + (long long)row * ld + kk * 16 + 8 * (lane >> 5));
}

// ---------------------------------------------------------------------------------------------
// dK / dV
// kPrefix: sequences may name an earlier sequence as their prefix.  The key block then also meets, after the
// queries of its own sequence (causal), every query of every sequence that names this one (no mask but the
// ends of the sequences): the tile stream is the concatenation of those, sequence by sequence.
template <bool kPrefix>
__global__ __launch_bounds__(256) void k_attn_bwd_dkv_mfma(AttnMfmaParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[4 * kStageBytes];
    const uint32_t lds0 = (uint32_t)(uintptr_t)ALCH_LDS(smem);
    // Work-groups are handed out in order of blockIdx.z first, so z counts the work down: a key block
    // with `rem` blocks of queries at or after it costs rem units, and the heaviest of all sequences
    // and heads start first (longest-processing-time-first keeps the last compute units busy).
    const int seq = blockIdx.y, kv = blockIdx.x;
    const int seq_start = p.cu[seq], len = p.cu[seq + 1] - seq_start;
    const int rem = (int)gridDim.z - (int)blockIdx.z, kb = (len + 127) / 128 - rem;
    if (kb < 0) return;
    const int lane = threadIdx.x & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int G = p.Hq / p.Hkv;
    const int j0 = kb * 128 + wave * 32;  // this wave's first key (index inside the sequence)

    // K, V fragments of the wave's 32 keys stay in registers
    const __bf16* Kb = p.K + (long long)seq_start * p.ldk + kv * kD;
    const __bf16* Vb = p.V + (long long)seq_start * p.ldk + kv * kD;
    bf16x8 kf[8], vf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        kf[kk] = global_frag_d(Kb, p.ldk, j0, len, kk, lane);
        vf[kk] = global_frag_d(Vb, p.ldk, j0, len, kk, lane);
    }
    f32x16 dK[4], dV[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) dK[n][e] = dV[n][e] = 0.f;

    const uint32_t lane_d = frag_d_lane(lane), lane_r0 = frag_rows_lane(lane, 0), lane_r1 = frag_rows_lane(lane, 1);
    uint32_t voff[4];
    tile_voffsets(voff, p.ldq, wave, lane);
    const int qt0 = (kb * 128) / kTileRows;
    const int nqt = (len + kTileRows - 1) / kTileRows - qt0;
    int n_it = G * nqt;
    if constexpr (kPrefix) {
        for (int c = seq + 1; c < p.n_seqs; ++c)
            if (p.prefix[c] == seq) n_it += G * ((p.cu[c + 1] - p.cu[c] + kTileRows - 1) / kTileRows);
    }
    const float sl2 = p.scale * kLog2e;

    // The tile stream: for the key block's own sequence and then (kPrefix) every sequence that names it as
    // prefix, for every query head of the group, the 64-query tiles qt_first .. qt_end-1 of that sequence.
    // Without prefixes the stream is ordered in two passes over the heads of the group: first the (at most two)
    // tiles of every head that meet the diagonal of the key block, which need the causal mask, then all the
    // others, which need none -- rows and keys past the end of the sequence are zero-filled by the loads, so
    // they contribute exactly nothing to rows that are stored.  n_mask iterations take the masked code.
    const int n_diag = kPrefix ? nqt : min(2, nqt);
    const int n_mask = kPrefix ? n_it : G * n_diag;
    struct Cursor {
        int c, row0, n;         // sequence of the queries, its first row in the batch, its length
        int qt_first, qt_end;   // its tiles that this key block meets in the current pass
        int h, qt;              // query head and tile of the current position
    };
    auto advance = [&](Cursor& q) {
        if (++q.qt < q.qt_end) return;
        q.qt = q.qt_first;
        if (++q.h < kv * G + G) return;
        q.h = kv * G;
        if constexpr (!kPrefix) {
            if (q.qt_first == qt0 && nqt > n_diag) {  // second pass: the tiles past the diagonal
                q.qt_first = q.qt = qt0 + n_diag;
                q.qt_end = qt0 + nqt;
            }
        }
        if constexpr (kPrefix) {
            int c = q.c + 1;
            while (c < p.n_seqs && !(p.prefix[c] == seq && p.cu[c + 1] > p.cu[c])) ++c;
            if (c < p.n_seqs) {
                q.c = c; q.row0 = p.cu[c]; q.n = p.cu[c + 1] - q.row0;
                q.qt_first = q.qt = 0; q.qt_end = (q.n + kTileRows - 1) / kTileRows;
            }
        }
        // (past the end of the stream the cursor wraps; its tiles are then loaded with zero extent)
    };
    // Software pipeline over the tile stream, four LDS stages (tile t in stage t & 3).  Entering iteration
    // `it`, of tile `it` (two blocks of 32 queries) the wave holds P, dS of block 0 packed to bf16 and the raw
    // scores S = Q K^T, dP = dO V^T of block 1.  The iteration waits for its own loads of tile it+1 (issued two
    // iterations ago) and meets the other waves (every wave is then past its reads of tile it-1, whose stage
    // receives tile it+3), then runs 64 matrix instructions in 16 groups of four:
    //   groups 0-7:  dV += P^T dO, dK += dS^T Q of block 0   |  S, dP of block 0 of tile it+1
    //   groups 8-15: the same for block 1                     |  S, dP of block 1 of tile it+1
    // Every matrix instruction is followed by its share of everything else, pinned in place (a wave issues in
    // order, so vector work only overlaps a matrix instruction that was issued before it): the six LDS reads of
    // the group two ahead, half of the exp/mask/dS work of two score elements (block 1 of tile `it` during
    // groups 0-7, block 0 of tile it+1 during groups 8-15), one of the nine direct-to-LDS loads of tile it+3,
    // the LSE / delta rows the coming groups need, and once per iteration the stream bookkeeping and the
    // buffer descriptors of the tile the next iteration loads.  Beyond the end of the stream the loads are
    // issued with zero extent: they move nothing and keep every wave's count of outstanding loads the same.
    f32x16 S1, dP1;         // raw scores of block 1 of the current tile
    bf16x8 pf0[2], dsf0[2]; // P, dS of block 0 of the current tile
    const int jl = j0 + (lane & 31);  // this lane's key
    const unsigned live_own = (unsigned)max(len - jl, 0);
    // P, dS of accumulator elements e0 .. e0+n-1 of one block, in place.  Element e is query row
    // i = i0 + 8*(e>>2) + 4*half + (e&3) against key column jl.  Pairs above the diagonal (jl > i) and rows
    // or keys past the end of the sequence get exponent -inf, i.e. p = 0 exactly: with rel = i - jl that
    // is one unsigned test, rel >= max(len - jl, 0).  Queries of a sequence that names this one as prefix
    // see every key: rel = i and the bound is that sequence's length (0 for a key past the end).
    // l, d: LSE and delta of the block's 16 rows of this lane.
    struct Meta { int ibase, sub; unsigned live; };  // first query row of a tile; what rel subtracts; the bound
    auto meta_of = [&](const Cursor& q) {
        Meta m;
        m.ibase = q.qt * kTileRows;
        if (!kPrefix || q.c == seq) { m.sub = jl; m.live = live_own; }
        else { m.sub = 0; m.live = jl < len ? (unsigned)q.n : 0u; }
        return m;
    };
    auto softmax_part = [&](f32x16& s, f32x16& dp, const f32x4 (&l)[4], const f32x4 (&d)[4], const Meta& m, int blk, int e0, int n) {
        const int rel0 = m.ibase + blk * 32 + 4 * half - (kPrefix ? m.sub : jl);
        const unsigned live = kPrefix ? m.live : live_own;
#pragma unroll
        for (int e = e0; e < e0 + n; ++e) {
            const unsigned rel = (unsigned)(rel0 + 8 * (e >> 2) + (e & 3));
            float arg = __builtin_fmaf(s[e], sl2, -l[e >> 2][e & 3]);
            arg = rel >= live ? -INFINITY : arg;
            const float pr = __builtin_amdgcn_exp2f(arg);
            s[e] = pr;
            dp[e] = pr * (dp[e] - d[e >> 2][e & 3]);
        }
    };
    auto load_row_scalars = [&](const char* stage, int ib, f32x4 (&l)[4], f32x4 (&d)[4]) {
        const float* lse_s = reinterpret_cast<const float*>(stage + 2 * kTileBytes);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            l[b] = *reinterpret_cast<const f32x4*>(lse_s + ib * 32 + 8 * b + 4 * half);
            d[b] = *reinterpret_cast<const f32x4*>(lse_s + 64 + ib * 32 + 8 * b + 4 * half);
        }
    };

    // Buffer descriptors of one tile's loads (Q rows, dO rows, and for the first two waves LSE / delta).
    struct LoadDesc { i32x4 q, dO, sc; };
    auto desc_of = [&](const Cursor& q, bool live) {
        const int rows = live ? q.n - q.qt * kTileRows : 0;
        const long long ext = rows > 0 ? ((long long)(rows - 1) * p.ldq + kD) * 2 : 0;
        const long long row = (long long)(q.row0 + q.qt * kTileRows);
        LoadDesc d;
        d.q = rsrc_of(p.Q + row * p.ldq + q.h * kD, ext);
        d.dO = rsrc_of(p.dO + row * p.ldq + q.h * kD, ext);
        d.sc = rsrc_of((wave == 0 ? p.lse2 : p.delta) + row * p.Hq + q.h,
                       (rows > 0 && wave < 2) ? ((long long)(rows - 1) * p.Hq + 1) * 4 : 0);
        return d;
    };
    // LDS address of the row-scalar load of this wave: LSE (wave 0), delta (wave 1); the other two waves issue the
    // same instruction with zero extent into the stage's padding, so every wave has nine loads per tile in flight
    const uint32_t sc_lds = 2 * kTileBytes + (wave < 2 ? (uint32_t)wave * 256u : 512u + (uint32_t)(wave - 2) * 256u);
    const uint32_t sc_voff = (uint32_t)(lane * p.Hq * 4);
    auto issue_tile = [&](const LoadDesc& d, uint32_t st) {
#pragma unroll
        for (int j = 0; j < 4; ++j) dma16(d.q, st + (uint32_t)(wave * 4 + j) * 1024u, voff[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) dma16(d.dO, st + kTileBytes + (uint32_t)(wave * 4 + j) * 1024u, voff[j]);
        dma4(d.sc, st + sc_lds, sc_voff);
    };
    // Four LDS stages, tile t in stage t & 3; iteration `it` works on tiles it and it+1 and loads tile it+3.
    Cursor q_ld{seq, seq_start, len, qt0, qt0 + n_diag, kv * G, qt0};
    Meta m_cur = meta_of(q_ld);
    issue_tile(desc_of(q_ld, 0 < n_it), lds0);
    advance(q_ld);
    Meta m_nxt = meta_of(q_ld);
    issue_tile(desc_of(q_ld, 1 < n_it), lds0 + kStageBytes);
    advance(q_ld);
    Meta m_nn = meta_of(q_ld);
    issue_tile(desc_of(q_ld, 2 < n_it), lds0 + 2 * kStageBytes);
    advance(q_ld);  // now at tile 3, the one iteration 0 loads
    Meta m_n3 = meta_of(q_ld);
    LoadDesc dsc = desc_of(q_ld, 3 < n_it);
    advance(q_ld);
    asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
    __syncthreads();
    f32x4 l1[4], d1[4];  // LSE, delta of block 1 of the current tile
    {   // tile 0: scores of both blocks, P and dS of block 0
        f32x16 S0, dP0;
#pragma unroll
        for (int e = 0; e < 16; ++e) S0[e] = dP0[e] = S1[e] = dP1[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            S0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(smem, lane_d, kk), kf[kk], S0, 0, 0, 0);
            dP0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(smem + kTileBytes, lane_d, kk), vf[kk], dP0, 0, 0, 0);
            S1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(smem + 32 * 256, lane_d, kk), kf[kk], S1, 0, 0, 0);
            dP1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(smem + kTileBytes + 32 * 256, lane_d, kk), vf[kk], dP1, 0, 0, 0);
        }
        f32x4 l[4], d[4];
        load_row_scalars(smem, 0, l, d);
        softmax_part(S0, dP0, l, d, m_cur, 0, 0, 16);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            pf0[ks] = pack8(S0, ks);
            dsf0[ks] = pack8(dP0, ks);
        }
        load_row_scalars(smem, 1, l1, d1);
    }

#define ALCH_SB __builtin_amdgcn_sched_barrier(0)
    struct Frags { bf16x8 rdo, rq, dq, ddo; };
    auto iteration = [&](auto masked_tag, int it) __attribute__((always_inline)) {
        constexpr bool kMasked = decltype(masked_tag)::value;
        const char* tq = smem + (uint32_t)(it & 3) * kStageBytes;
        const char* tdo = tq + kTileBytes;
        const char* nq = smem + (uint32_t)((it + 1) & 3) * kStageBytes;
        const char* ndo = nq + kTileBytes;
        const uint32_t st3 = lds0 + (uint32_t)((it + 3) & 3) * kStageBytes;

        ALCH_SB;
        asm volatile("s_waitcnt vmcnt(9)" ::: "memory");  // tile it+1 has landed (tile it+2 may still be on its way)
        __syncthreads();
        ALCH_SB;

        f32x4 ln[4], dn[4];  // LSE, delta of block 0 of the next tile
        Frags fr[3];
        auto ld_rdo = [&](int g) { fr[g % 3].rdo = lds_frag_rows(tdo + (g >> 3) * 32 * 256, lane_r0, lane_r1, (g >> 2) & 1, g & 3); };
        auto ld_rq = [&](int g) { fr[g % 3].rq = lds_frag_rows(tq + (g >> 3) * 32 * 256, lane_r0, lane_r1, (g >> 2) & 1, g & 3); };
        auto ld_d = [&](int g) {
            const int kk = ((g >> 2) & 1) * 4 + (g & 3);
            fr[g % 3].dq = lds_frag_d(nq + (g >> 3) * 32 * 256, lane_d, kk);
            fr[g % 3].ddo = lds_frag_d(ndo + (g >> 3) * 32 * 256, lane_d, kk);
        };
        ld_rdo(0); ld_rq(0); ld_d(0);
        ld_rdo(1); ld_rq(1); ld_d(1);
        f32x16 Sn0, dPn0, Sn1, dPn1;  // scores of the next tile
        bf16x8 pf1[2], dsf1[2], pfn[2], dsfn[2];
        Meta m_n4;
        LoadDesc dsc_next;
        // One element of the softmax gradient in two halves, each pinned where it is written so that it is issued
        // between two matrix instructions: h1 = masked exponent -> probability, h2 = dS = p (dP - delta).
        {
            auto sm_h1 = [&](f32x16& sc, const f32x4 (&l)[4], const Meta& m, int blk, int e) {
                float arg = __builtin_fmaf(sc[e], sl2, -l[e >> 2][e & 3]);
                if constexpr (kMasked) {
                    const int rel0 = m.ibase + blk * 32 + 4 * half - (kPrefix ? m.sub : jl);
                    const unsigned live = kPrefix ? m.live : live_own;
                    const unsigned rel = (unsigned)(rel0 + 8 * (e >> 2) + (e & 3));
                    arg = rel >= live ? -INFINITY : arg;
                }
                float pr = __builtin_amdgcn_exp2f(arg);
                asm volatile("" : "+v"(pr));
                sc[e] = pr;
            };
            auto sm_h2 = [&](const f32x16& sc, f32x16& dp, const f32x4 (&d)[4], int e) {
                float t = sc[e] * (dp[e] - d[e >> 2][e & 3]);
                asm volatile("" : "+v"(t));
                dp[e] = t;
            };
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int ib = g >> 3, ks = (g >> 2) & 1, nb = g & 3, kk = ks * 4 + nb;
                const int ea = ib == 0 ? 2 * g : 2 * (g - 8), eb = ea + 1;
                const Frags& f = fr[g % 3];
                // slot 0
                if (g + 2 < 16) ld_rdo(g + 2);
                if (ib == 0) sm_h1(S1, l1, m_cur, 1, ea); else sm_h1(Sn0, ln, m_nxt, 0, ea);
                ALCH_SB;
                dV[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ib == 0 ? pf0[ks] : pf1[ks], f.rdo, dV[nb], 0, 0, 0);
                ALCH_SB;
                // slot 1
                if (g + 2 < 16) ld_rq(g + 2);
                if (ib == 0) sm_h1(S1, l1, m_cur, 1, eb); else sm_h1(Sn0, ln, m_nxt, 0, eb);
                ALCH_SB;
                dK[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ib == 0 ? dsf0[ks] : dsf1[ks], f.rq, dK[nb], 0, 0, 0);
                ALCH_SB;
                // slot 2
                if (g + 2 < 16) ld_d(g + 2);
                if (ib == 0) { sm_h2(S1, dP1, d1, ea); sm_h2(S1, dP1, d1, eb); }
                else { sm_h2(Sn0, dPn0, dn, ea); sm_h2(Sn0, dPn0, dn, eb); }
                ALCH_SB;
                if (g == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) Sn0[e] = dPn0[e] = 0.f;
                }
                if (g == 8) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) Sn1[e] = dPn1[e] = 0.f;
                }
                if (ib == 0) Sn0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.dq, kf[kk], Sn0, 0, 0, 0);
                else Sn1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.dq, kf[kk], Sn1, 0, 0, 0);
                ALCH_SB;
                // slot 3: the loads of tile it+3, the row scalars the next groups need, the stream bookkeeping, packs
                if (g < 4) dma16(dsc.q, st3 + (uint32_t)(wave * 4 + g) * 1024u, voff[g & 3]);
                else if (g < 8) dma16(dsc.dO, st3 + kTileBytes + (uint32_t)(wave * 4 + g - 4) * 1024u, voff[g & 3]);
                else if (g == 8) dma4(dsc.sc, st3 + sc_lds, sc_voff);
                if (g < 4) {       // LSE, delta of block 0 of tile it+1 (used from group 8 on)
                    const float* sc_n = reinterpret_cast<const float*>(nq + 2 * kTileBytes);
                    ln[g] = *reinterpret_cast<const f32x4*>(sc_n + 8 * g + 4 * half);
                    dn[g] = *reinterpret_cast<const f32x4*>(sc_n + 64 + 8 * g + 4 * half);
                }
                if (g >= 12) {     // LSE, delta of block 1 of tile it+1 (used by the next iteration's groups 0-7)
                    const float* sc_n = reinterpret_cast<const float*>(nq + 2 * kTileBytes);
                    l1[g - 12] = *reinterpret_cast<const f32x4*>(sc_n + 32 + 8 * (g - 12) + 4 * half);
                    d1[g - 12] = *reinterpret_cast<const f32x4*>(sc_n + 64 + 32 + 8 * (g - 12) + 4 * half);
                }
                if (g == 9) {      // position and descriptors of tile it+4, which the next iteration loads
                    m_n4 = meta_of(q_ld);
                    dsc_next = desc_of(q_ld, it + 4 < n_it);
                    advance(q_ld);
                }
                if (g == 3) { pf1[0] = pack8(S1, 0); dsf1[0] = pack8(dP1, 0); asm volatile("" : "+v"(pf1[0]), "+v"(dsf1[0])); }
                if (g == 7) { pf1[1] = pack8(S1, 1); dsf1[1] = pack8(dP1, 1); asm volatile("" : "+v"(pf1[1]), "+v"(dsf1[1])); }
                if (g == 11) { pfn[0] = pack8(Sn0, 0); dsfn[0] = pack8(dPn0, 0); asm volatile("" : "+v"(pfn[0]), "+v"(dsfn[0])); }
                if (g == 15) { pfn[1] = pack8(Sn0, 1); dsfn[1] = pack8(dPn0, 1); asm volatile("" : "+v"(pfn[1]), "+v"(dsfn[1])); }
                ALCH_SB;
                if (ib == 0) dPn0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ddo, vf[kk], dPn0, 0, 0, 0);
                else dPn1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ddo, vf[kk], dPn1, 0, 0, 0);
                ALCH_SB;
            }
        }
        // hand over to the next iteration
        S1 = Sn1; dP1 = dPn1;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) { pf0[ks] = pfn[ks]; dsf0[ks] = dsfn[ks]; }
        m_cur = m_nxt; m_nxt = m_nn; m_nn = m_n3; m_n3 = m_n4;
        dsc = dsc_next;
    };
    {
        int it = 0;
        for (; it < n_mask && it < n_it; ++it) iteration(std::true_type{}, it);
        for (; it < n_it; ++it) iteration(std::false_type{}, it);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // accumulator element e of block nb: key row j0 + 8*(e>>2) + 4*half + (e&3), column nb*32 + (lane&31)
    if (p.rope_log2_base > 0.f) rope_backward_rows(dK, p, seq_start, j0, len, lane);
    __bf16* dKb = p.dK + (long long)seq_start * p.ldo + kv * kD;
    __bf16* dVb = p.dV + (long long)seq_start * p.ldo + kv * kD;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int j = j0 + 8 * (e >> 2) + 4 * half + (e & 3);
            if (j < len) {
                const long long off = (long long)j * p.ldo + nb * 32 + (lane & 31);
                dKb[off] = (__bf16)(dK[nb][e] * p.scale);
                dVb[off] = (__bf16)dV[nb][e];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// dQ
__global__ __launch_bounds__(256, 2) void k_attn_bwd_dq_mfma(AttnMfmaParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];
    const uint32_t lds0 = (uint32_t)(uintptr_t)ALCH_LDS(smem);
    const int seq = blockIdx.y, h = blockIdx.x;
    const int seq_start = p.cu[seq], len = p.cu[seq + 1] - seq_start;
    // heaviest (last) query blocks of every sequence and head first: blockIdx.z is the slowest index
    const int qb = (int)gridDim.z - 1 - (int)blockIdx.z;
    if (qb * 128 >= len) return;
    const int lane = threadIdx.x & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kv = h / (p.Hq / p.Hkv);
    const int i0 = qb * 128 + wave * 32;  // this wave's first query

    const uint32_t lane_d = frag_d_lane(lane), lane_r0 = frag_rows_lane(lane, 0), lane_r1 = frag_rows_lane(lane, 1);
    uint32_t voff[4];
    tile_voffsets(voff, p.ldk, wave, lane);
    // key tiles: all tiles of the prefix sequence (if any), then own tiles 0 .. the last one that holds a
    // key <= the work-group's last query
    const int pre = p.prefix ? p.prefix[seq] : -1;
    const int pre_start = pre >= 0 ? p.cu[pre] : 0, pre_len = pre >= 0 ? p.cu[pre + 1] - pre_start : 0;
    const int npt = (pre_len + kTileRows - 1) / kTileRows;
    const int last_q = min(qb * 128 + 127, len - 1);
    const int n_it = npt + last_q / kTileRows + 1;
    const float sl2 = p.scale * kLog2e;
    // Buffer descriptors of a tile from scalar arithmetic alone: base of the sequence's K / V plus the tile's byte
    // offset, extent = what is left of the sequence (rows past its end read as zero), both below 2 GiB.
    const long long kv_off = (long long)kv * kD;
    const unsigned long long baseK_own = reinterpret_cast<unsigned long long>(p.K + (long long)seq_start * p.ldk + kv_off);
    const unsigned long long baseV_own = reinterpret_cast<unsigned long long>(p.V + (long long)seq_start * p.ldk + kv_off);
    const unsigned long long baseK_pre = reinterpret_cast<unsigned long long>(p.K + (long long)pre_start * p.ldk + kv_off);
    const unsigned long long baseV_pre = reinterpret_cast<unsigned long long>(p.V + (long long)pre_start * p.ldk + kv_off);
    const unsigned tile_bytes = (unsigned)(kTileRows * p.ldk * 2);   // distance of two tiles
    struct TileSrc { i32x4 k, v; };
    auto desc = [&](unsigned long long base, int rows) {
        const unsigned n = rows > 0 ? (unsigned)(((long long)(min(rows, kTileRows) - 1) * p.ldk + kD) * 2) : 0u;
        i32x4 r;
        r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
        r[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(base >> 32) & 0xffffu));
        r[2] = __builtin_amdgcn_readfirstlane((int)n);
        r[3] = 0x00020000;
        return r;
    };
    auto tile_src = [&](int it) {
        const bool in_pre = it < npt;
        const int tile = in_pre ? it : it - npt;
        const int rows = it < n_it ? (in_pre ? pre_len : len) - tile * kTileRows : 0;  // past the last tile: nothing moves
        const unsigned long long off = (unsigned long long)tile * tile_bytes;
        TileSrc t;
        t.k = desc((in_pre ? baseK_pre : baseK_own) + off, rows);
        t.v = desc((in_pre ? baseV_pre : baseV_own) + off, rows);
        return t;
    };
    // load j (0..7) of a wave's share of tile `it`: four 1 KB pieces of the K tile, four of the V tile
    auto issue_piece = [&](const TileSrc& t, int it, int j) {
        const uint32_t st = lds0 + (uint32_t)(it & 1) * kStageBytes + (j < 4 ? 0u : (uint32_t)kTileBytes);
        dma16(j < 4 ? t.k : t.v, st + (uint32_t)(wave * 4 + (j & 3)) * 1024u, voff[j & 3]);
    };
    {   // the first tile is on its way while the Q, dO and O fragments below are fetched
        const TileSrc t0 = tile_src(0);
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_piece(t0, 0, j);
    }
    const __bf16* Qb = p.Q + (long long)seq_start * p.ldq + h * kD;
    const __bf16* dOb = p.dO + (long long)seq_start * p.ldq + h * kD;
    bf16x8 qf[8], gf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        qf[kk] = global_frag_d(Qb, p.ldq, i0, len, kk, lane);
        gf[kk] = global_frag_d(dOb, p.ldq, i0, len, kk, lane);
    }
    const int i = i0 + (lane & 31);  // this lane's query (accumulator column)
    const bool i_ok = i < len;
    const float lse2 = i_ok ? p.LSE[(long long)(seq_start + i) * p.Hq + h] * kLog2e : 0.f;
    if (i_ok && half == 0) p.lse2[(long long)(seq_start + i) * p.Hq + h] = lse2;
    // delta_i = sum_d dO[i,d] O[i,d]: each lane holds 64 of the 128 elements of its query's dO row
    float del = 0.f;
    {
        const __bf16* Ob = p.O + (long long)seq_start * p.ldq + h * kD;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 of = global_frag_d(Ob, p.ldq, i0, len, kk, lane);
#pragma unroll
            for (int e = 0; e < 8; ++e) del += (float)of[e] * (float)gf[kk][e];
        }
        del += __shfl_xor(del, 32, 64);
        if (i_ok && half == 0) p.delta[(long long)(seq_start + i) * p.Hq + h] = del;
    }
    const float ndel = -del;
    f32x16 dQ[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) dQ[n][e] = 0.f;

    for (int it = 0; it < n_it; ++it) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        {   // the loads of tile it+1 (two waves share a SIMD: while this one queues its loads the other computes)
            const TileSrc tn = tile_src(it + 1);
#pragma unroll
            for (int j = 0; j < 8; ++j) issue_piece(tn, it + 1, j);
        }
        const char* tk = smem + (it & 1) * kStageBytes;
        const char* tv = tk + kTileBytes;
        // keys of this tile count from 0 inside their own sequence; key j is visible to query i when
        // j <= lim: the last prefix key for a prefix tile, i itself (the diagonal) for an own tile
        const bool in_pre = it < npt;
        const int jt = (in_pre ? it : it - npt) * kTileRows;
        const int lim = in_pre ? pre_len - 1 : i, lim0 = in_pre ? pre_len - 1 : i0;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int j0 = jt + jb * 32;
            // a 32-key block wholly above this wavefront's diagonal contributes nothing: skipped (the other
            // wavefronts of the work-group, further down the diagonal, still need the tile)
            if (!in_pre && j0 > i0 + 31) continue;
            const char* bk = tk + jb * 32 * 256;
            const char* bv = tv + jb * 32 * 256;
            // transposed: rows = keys, columns = queries.  dP starts from -delta (every element of a lane belongs
            // to the lane's query), so the accumulator comes out as dP - delta
            f32x16 St, dPt;
#pragma unroll
            for (int e = 0; e < 16; ++e) { St[e] = 0.f; dPt[e] = ndel; }
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                St = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(bk, lane_d, kk), qf[kk], St, 0, 0, 0);
                dPt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(bv, lane_d, kk), gf[kk], dPt, 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(St[e], sl2, -lse2));
                dPt[e] = pr * dPt[e];
            }
            if (!i_ok || j0 + 31 > lim0) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int j = j0 + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (!i_ok || j > lim) dPt[e] = 0.f;
                }
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                // left operand dS[i][j]: row i = lane&31 (this lane's query), k <-> key rows of the accumulator
                const bf16x8 dsf = pack8(dPt, ks);
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    dQ[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf, lds_frag_rows(bk, lane_r0, lane_r1, ks, nb), dQ[nb], 0, 0, 0);
            }
        }
    }

    if (p.rope_log2_base > 0.f) rope_backward_rows(dQ, p, seq_start, i0, len, lane);
    __bf16* dQb = p.dQ + (long long)seq_start * p.ldo + h * kD;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int ii = i0 + 8 * (e >> 2) + 4 * half + (e & 3);
            if (ii < len) dQb[(long long)ii * p.ldo + nb * 32 + (lane & 31)] = (__bf16)(dQ[nb][e] * p.scale);
        }
}

// ---------------------------------------------------------------------------------------------
// forward: O = softmax_causal(Q K^T / sqrt(D)) V and LSE, the step of the prefill that produces the
// O and LSE members of the record.  A work-group owns 128 queries of one (sequence, head), 32 per
// wavefront with their Q fragments in registers, and streams 64-key tiles of K and V through LDS.
// Scores are formed transposed (rows = keys, columns = queries) so that a lane owns one query: its
// running maximum, normaliser and the rescaling of its output column are per-lane scalars, and P
// in the accumulator layout is directly the right operand of O^T += V^T P^T.
struct AttnFwdParams {
    const __bf16 *Q, *K, *V;
    __bf16* O;
    float* LSE;
    const int* cu;
    const int* prefix;  // as in the backward
    int seq_begin;      // first sequence whose queries are computed
    int Hq, Hkv;
    long long ldq, ldk;
    float scale;
};

__global__ __launch_bounds__(256, 2) void k_attn_fwd_mfma(AttnFwdParams p) {
    __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];
    const uint32_t lds0 = (uint32_t)(uintptr_t)ALCH_LDS(smem);
    const int seq = p.seq_begin + blockIdx.y, h = blockIdx.x;
    const int seq_start = p.cu[seq], len = p.cu[seq + 1] - seq_start;
    // heaviest (last) query blocks of every sequence and head first: blockIdx.z is the slowest index
    const int qb = (int)gridDim.z - 1 - (int)blockIdx.z;
    if (qb * 128 >= len) return;
    const int lane = threadIdx.x & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kv = h / (p.Hq / p.Hkv);
    const int i0 = qb * 128 + wave * 32;

    const __bf16* Qb = p.Q + (long long)seq_start * p.ldq + h * kD;
    bf16x8 qf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = global_frag_d(Qb, p.ldq, i0, len, kk, lane);
    const int i = i0 + (lane & 31);
    f32x16 Ot[4];  // O^T: block nb holds d = nb*32 + 8b + 4*half + r (register 4b+r) of query i
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) Ot[n][e] = 0.f;
    float m2 = -INFINITY, l = 0.f;  // running max (log2 domain) and normaliser of this lane's half of the keys

    const uint32_t lane_d = frag_d_lane(lane), lane_r0 = frag_rows_lane(lane, 0), lane_r1 = frag_rows_lane(lane, 1);
    uint32_t voff[4];
    tile_voffsets(voff, p.ldk, wave, lane);
    // key tiles: all tiles of the prefix sequence (if any), then the own tiles up to the diagonal; one
    // running maximum and normaliser cover both, so O and LSE are those of the joint softmax
    const int pre = p.prefix ? p.prefix[seq] : -1;
    const int pre_start = pre >= 0 ? p.cu[pre] : 0, pre_len = pre >= 0 ? p.cu[pre + 1] - pre_start : 0;
    const int npt = (pre_len + kTileRows - 1) / kTileRows;
    const int last_q = min(qb * 128 + 127, len - 1);
    const int n_it = npt + last_q / kTileRows + 1;
    const float sl2 = p.scale * kLog2e;

    auto issue = [&](int it) {
        const bool in_pre = it < npt;
        const int row_first = (in_pre ? it : it - npt) * kTileRows;
        const int rows_valid = (in_pre ? pre_len : len) - row_first;
        const long long row = (long long)((in_pre ? pre_start : seq_start) + row_first);
        const uint32_t st = lds0 + (uint32_t)(it & 1) * kStageBytes;
        issue_rows_tile(p.K + row * p.ldk + kv * kD, p.ldk, rows_valid, st, wave, voff);
        issue_rows_tile(p.V + row * p.ldk + kv * kD, p.ldk, rows_valid, st + kTileBytes, wave, voff);
    };

    issue(0);
    for (int it = 0; it < n_it; ++it) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (it + 1 < n_it) issue(it + 1);
        const char* tk = smem + (it & 1) * kStageBytes;
        const char* tv = tk + kTileBytes;
        const bool in_pre = it < npt;
        const int jt = (in_pre ? it : it - npt) * kTileRows;  // first key of the tile inside its own sequence
        const int lim = in_pre ? pre_len - 1 : i;             // last key of the tile's sequence this query sees
        // (a tile wholly above this wave's diagonal is computed and fully masked: p = 0, alpha = 1)
        f32x16 St[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) St[jb][e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                St[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_d(tk + jb * 32 * 256, lane_d, kk), qf[kk], St[jb], 0, 0, 0);
        }
        // scores in the log2 domain, masked (key j = jt + jb*32 + 8b + 4*half + r must satisfy j <= lim)
        const bool need_mask = jt + 63 > (in_pre ? pre_len - 1 : i0);
        float mx = m2;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float sv = St[jb][e] * sl2;
                if (need_mask) {
                    const int j = jt + jb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (j > lim) sv = -INFINITY;
                }
                St[jb][e] = sv;
                mx = fmaxf(mx, sv);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // both halves of the wave share the query
        const float alpha = __builtin_amdgcn_exp2f(m2 - mx);  // 0 on the first tile (m2 = -inf), keys 0.. always valid
        m2 = mx;
        float sum = 0.f;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float pr = __builtin_amdgcn_exp2f(St[jb][e] - mx);
                St[jb][e] = pr;
                sum += pr;
            }
        l = l * alpha + sum;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) Ot[n][e] *= alpha;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 pf = pack8(St[jb], ks);  // right operand P^T: column = this lane's query, k <-> key rows
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    Ot[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_rows(tv + jb * 32 * 256, lane_r0, lane_r1, ks, nb), pf, Ot[nb], 0, 0, 0);
            }
    }
    l += __shfl_xor(l, 32, 64);
    if (i < len) {
        const float inv = 1.f / l;
        __bf16* orow = p.O + (long long)(seq_start + i) * p.ldq + h * kD;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (__bf16)(Ot[nb][4 * b + r] * inv);
                *reinterpret_cast<bf16x4*>(orow + nb * 32 + 8 * b + 4 * half) = o;
            }
        if (half == 0) p.LSE[(long long)(seq_start + i) * p.Hq + h] = (m2 + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
}

bool attn_mfma_supported(const AttnArgs& a) {
    return a.dtype == ALCH_BF16 && a.D == kD && a.T > 0 && a.ld_dqkv % 8 == 0 && aligned16(a.Q) && aligned16(a.K) &&
           aligned16(a.V) && aligned16(a.dO) && aligned16(a.O);
}

int launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t stream) {
    AttnMfmaParams p;
    p.Q = (const __bf16*)a.Q; p.K = (const __bf16*)a.K; p.V = (const __bf16*)a.V; p.dO = (const __bf16*)a.dO;
    p.O = (const __bf16*)a.O; p.LSE = a.LSE; p.delta = a.delta; p.lse2 = a.delta + (size_t)a.T * a.Hq;
    p.positions = a.positions; p.rope_log2_base = a.rope_base > 0.f ? log2f(a.rope_base) : 0.f;
    p.dQ = (__bf16*)a.dQ; p.dK = (__bf16*)a.dK; p.dV = (__bf16*)a.dV;
    p.cu = a.cu_seqlens; p.prefix = a.prefix; p.n_seqs = a.n_seqs; p.Hq = a.Hq; p.Hkv = a.Hkv;
    p.ldq = (long long)a.Hq * a.D; p.ldk = (long long)a.Hkv * a.D; p.ldo = a.ld_dqkv;
    p.scale = 1.0f / sqrtf((float)a.D);
    const int nb = ceil_div(a.max_seqlen, 128);
    if (nb <= 0 || a.n_seqs <= 0) return ALCH_OK;
    if (nb > 65535 || a.n_seqs > 65535) return fail(ALCH_ERR_UNSUPPORTED, "attention: more than 65535 sequences or 128-token blocks");
    k_attn_bwd_dq_mfma<<<dim3(a.Hq, a.n_seqs, nb), 256, 0, stream>>>(p);   // also writes delta
    if (a.prefix)
        k_attn_bwd_dkv_mfma<true><<<dim3(a.Hkv, a.n_seqs, nb), 256, 0, stream>>>(p);
    else
        k_attn_bwd_dkv_mfma<false><<<dim3(a.Hkv, a.n_seqs, nb), 256, 0, stream>>>(p);
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

int launch_attn_fwd(alch_dtype dt, const void* Q, const void* K, const void* V, void* O, float* LSE, int T,
                    int n_seqs, int max_seqlen, const int* cu_seqlens, const int* cu_seqlens_host, const int* prefix,
                    const int* prefix_host, int seq_begin, int Hq, int Hkv, int D, hipStream_t stream) {
    if (seq_begin >= n_seqs) return ALCH_OK;
    const double pairs = attn_pairs(n_seqs - seq_begin, cu_seqlens_host + seq_begin, nullptr) +
                         (attn_pairs(n_seqs, cu_seqlens_host, prefix_host) - attn_pairs(n_seqs, cu_seqlens_host, nullptr));
    TraceScope ts(kTraceAttnFwd, 4.0 * D * Hq * pairs, 0.0, stream);
    if (dt == ALCH_BF16 && D == kD && T > 0 && aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(O)) {
        AttnFwdParams p;
        p.Q = (const __bf16*)Q; p.K = (const __bf16*)K; p.V = (const __bf16*)V; p.O = (__bf16*)O; p.LSE = LSE;
        p.cu = cu_seqlens; p.prefix = prefix; p.seq_begin = seq_begin;
        p.Hq = Hq; p.Hkv = Hkv; p.ldq = (long long)Hq * D; p.ldk = (long long)Hkv * D;
        p.scale = 1.0f / sqrtf((float)D);
        const int nb = ceil_div(max_seqlen, 128);
        if (nb <= 0 || n_seqs <= 0) return ALCH_OK;
        if (nb > 65535 || n_seqs > 65535) return fail(ALCH_ERR_UNSUPPORTED, "attention: more than 65535 sequences or 128-token blocks");
        k_attn_fwd_mfma<<<dim3(Hq, n_seqs - seq_begin, nb), 256, 0, stream>>>(p);
        ALCH_HIP_TRY(hipGetLastError());
        return ALCH_OK;
    }
    return launch_attn_fwd_generic(dt, Q, K, V, O, LSE, T, n_seqs, cu_seqlens, cu_seqlens_host, prefix, seq_begin, Hq, Hkv, D, stream);
}

}  // namespace alch
