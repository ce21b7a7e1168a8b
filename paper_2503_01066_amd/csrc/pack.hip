// Capture/pack: mask scan and row gather (Section 4.1 of the paper: only the tokens of the
// prefill that are to be trained on are recorded; Section 5: one record per layer).
//
// The scan is one single-work-group kernel for batches of up to 262,144 tokens, and beyond that four small
// kernels over the byte mask (per-block popcount, scan of the block counts, index fill, per-sequence counts)
// with the block counts in caller-provided scratch; the gather runs one work-group per kept row,
// moving 16 bytes per lane per access.  Everything is bit-exact and
// deterministic: the output order is the ascending token order.
#include "common.h"
#include "kernels.h"

namespace alch {

static constexpr int kTokPerThread = 16;
static constexpr int kScanThreads = 256;
static constexpr int kTokPerBlock = kTokPerThread * kScanThreads;  // 4096

__device__ __forceinline__ int nonzero_bytes16(const uint8_t* __restrict__ mask, int t0, int T, uint32_t& bits) {
    // bits: bit i set <=> mask[t0+i] != 0 (tokens beyond T count as dropped)
    bits = 0;
    if (t0 + kTokPerThread <= T) {
        uint4 v = *reinterpret_cast<const uint4*>(mask + t0);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if ((w[i] >> (8 * b)) & 0xffu) bits |= 1u << (4 * i + b);
    } else {
        for (int i = 0; i < kTokPerThread; ++i)
            if (t0 + i < T && mask[t0 + i] != 0) bits |= 1u << i;
    }
    return __popc(bits);
}

__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan of one int per thread over a block of kScanThreads; returns the exclusive
// prefix, writes the block total to `total`.
__device__ __forceinline__ int block_exclusive_scan(int v, int& total) {
    __shared__ int wave_sum[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = wave_inclusive_scan(v);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        int s = wave_sum[w];
        if (w < wave) before += s;
        tot += s;
    }
    total = tot;
    __syncthreads();
    return before + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void k_pack_count(const uint8_t* __restrict__ mask, int T,
                                                             int* __restrict__ block_counts) {
    uint32_t bits;
    int c = nonzero_bytes16(mask, (blockIdx.x * kScanThreads + threadIdx.x) * kTokPerThread, T, bits);
    int total;
    block_exclusive_scan(c, total);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

// One block: exclusive scan of the block counts in place -> block offsets; n_kept and overflow flag.
__global__ __launch_bounds__(kScanThreads) void k_pack_scan_blocks(int* __restrict__ block_counts, int nblocks,
                                                                   int* __restrict__ n_kept_and_status,
                                                                   long long capacity) {
    int carry = 0;
    for (int base = 0; base < nblocks; base += kScanThreads) {
        int i = base + threadIdx.x;
        int v = i < nblocks ? block_counts[i] : 0;
        int total;
        int ex = block_exclusive_scan(v, total);
        if (i < nblocks) block_counts[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) {
        n_kept_and_status[0] = carry;
        n_kept_and_status[1] = (long long)carry > capacity ? 1 : 0;
    }
}

__global__ __launch_bounds__(kScanThreads) void k_pack_fill(const uint8_t* __restrict__ mask, int T,
                                                            const int* __restrict__ block_offsets,
                                                            int* __restrict__ kept_index, long long capacity) {
    uint32_t bits;
    const int t0 = (blockIdx.x * kScanThreads + threadIdx.x) * kTokPerThread;
    int c = nonzero_bytes16(mask, t0, T, bits);
    int total;
    long long pos = (long long)block_offsets[blockIdx.x] + block_exclusive_scan(c, total);
    while (bits) {
        int i = __ffs(bits) - 1;
        bits &= bits - 1;
        if (pos < capacity) kept_index[pos] = t0 + i;
        ++pos;
    }
}

// One wave per sequence boundary: cu_kept[s] = kept tokens before token cu_seqlens[s].
__global__ __launch_bounds__(64) void k_pack_cu(const uint8_t* __restrict__ mask, const int* __restrict__ cu_seqlens,
                                                int n_bounds, const int* __restrict__ block_offsets, int nblocks,
                                                const int* __restrict__ n_kept_and_status,
                                                int* __restrict__ cu_kept) {
    const int s = blockIdx.x;
    if (s >= n_bounds) return;
    const int end = cu_seqlens[s];
    const int blk = end / kTokPerBlock;
    int count = 0;
    for (int t = blk * kTokPerBlock + threadIdx.x; t < end; t += 64) count += mask[t] != 0;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) count += __shfl_down(count, d, 64);
    if (threadIdx.x == 0) cu_kept[s] = (blk < nblocks ? block_offsets[blk] : n_kept_and_status[0]) + count;
}

// ---- the whole scan in one launch, for batches of up to kOneLaunchTokens tokens ------------------------
// One work-group of 1024 threads; thread i owns the tokens [i * chunk, (i + 1) * chunk) with chunk a multiple
// of 16 (<= 256): it counts its kept tokens, the block scans the 1024 counts, and the thread writes the indices
// of its kept tokens; then one thread per sequence boundary forms cu_kept from the scanned counts.  A prefill
// batch of the paper's sizes (tens of thousands of tokens) is a mask of tens of kilobytes: four launches of the
// general path cost more than the work.
static constexpr int kOneLaunchThreads = 1024;
static constexpr int kOneLaunchTokens = kOneLaunchThreads * 256;

__global__ __launch_bounds__(kOneLaunchThreads) void k_pack_scan_one(const uint8_t* __restrict__ mask, int T, int chunk,
                                                                      const int* __restrict__ cu_seqlens, int n_bounds,
                                                                      int* __restrict__ kept_index, int* __restrict__ cu_kept,
                                                                      int* __restrict__ n_kept_and_status, long long capacity) {
    __shared__ int prefix[kOneLaunchThreads];            // kept tokens before each thread's chunk
    __shared__ int wave_sum[kOneLaunchThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t_begin = tid * chunk;
    int count = 0;
    for (int t0 = t_begin; t0 < t_begin + chunk && t0 < T; t0 += kTokPerThread) {
        uint32_t bits;
        count += nonzero_bytes16(mask, t0, T, bits);
    }
    const int inc = wave_inclusive_scan(count);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kOneLaunchThreads / 64; ++w) {
        const int sw = wave_sum[w];
        if (w < wave) before += sw;
        total += sw;
    }
    const int ex = before + inc - count;
    prefix[tid] = ex;
    if (tid == 0) {
        n_kept_and_status[0] = total;
        n_kept_and_status[1] = (long long)total > capacity ? 1 : 0;
    }
    long long pos = ex;
    for (int t0 = t_begin; t0 < t_begin + chunk && t0 < T; t0 += kTokPerThread) {
        uint32_t bits;
        nonzero_bytes16(mask, t0, T, bits);
        while (bits) {
            const int i = __ffs(bits) - 1;
            bits &= bits - 1;
            if (pos < capacity) kept_index[pos] = t0 + i;
            ++pos;
        }
    }
    __syncthreads();
    for (int s = tid; s < n_bounds; s += kOneLaunchThreads) {
        const int end = cu_seqlens[s];
        const int owner = end / chunk;  // thread whose chunk holds token `end` (>= 1024 only for end == T at full chunks)
        int c = owner < kOneLaunchThreads ? prefix[owner] : total;
        for (int t = owner * chunk; t < end; ++t) c += mask[t] != 0;
        cu_kept[s] = c;
    }
}

// ---- gather ---------------------------------------------------------------------------

struct GatherArgs {
    const char* src[kMaxStreamsPerLaunch];
    char* dst[kMaxStreamsPerLaunch];
    unsigned long long row_bytes[kMaxStreamsPerLaunch];
    unsigned long long src_stride[kMaxStreamsPerLaunch];
    int n;
};

// One work-group per kept row (the grid is sized for the most rows the call can produce; work-groups
// beyond n_kept leave at once).  Letting the hardware dispatcher hand out rows measured faster than a
// persistent grid: the rows of the wide streams are long enough to keep every lane busy.
template <typename V>
__global__ __launch_bounds__(256) void k_pack_gather(GatherArgs a, const int* __restrict__ kept_index,
                                                     const int* __restrict__ n_kept_and_status,
                                                     long long capacity) {
    long long n_rows = n_kept_and_status[0];
    if (n_rows > capacity) n_rows = capacity;
    constexpr unsigned long long kStep = 256ull * sizeof(V);
    for (long long r = blockIdx.x; r < n_rows; r += gridDim.x) {
        const long long t = kept_index[r];
        for (int k = 0; k < a.n; ++k) {
            const unsigned long long rb = a.row_bytes[k];
            const char* __restrict__ s = a.src[k] + (unsigned long long)t * a.src_stride[k];
            char* __restrict__ d = a.dst[k] + (unsigned long long)r * rb;
            unsigned long long off = (unsigned long long)threadIdx.x * sizeof(V);
            // two independent accesses in flight per lane; non-temporal both ways (nothing is reused)
            for (; off + kStep < rb; off += 2 * kStep) {
                V v0 = __builtin_nontemporal_load(reinterpret_cast<const V*>(s + off));
                V v1 = __builtin_nontemporal_load(reinterpret_cast<const V*>(s + off + kStep));
                __builtin_nontemporal_store(v0, reinterpret_cast<V*>(d + off));
                __builtin_nontemporal_store(v1, reinterpret_cast<V*>(d + off + kStep));
            }
            for (; off < rb; off += kStep) {
                V v = __builtin_nontemporal_load(reinterpret_cast<const V*>(s + off));
                __builtin_nontemporal_store(v, reinterpret_cast<V*>(d + off));
            }
        }
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

size_t pack_workspace_bytes(int total_tokens) {
    int nblocks = ceil_div(total_tokens > 0 ? total_tokens : 1, kTokPerBlock);
    return round_up((size_t)nblocks * sizeof(int), 256) + 256;
}

int launch_pack(const uint8_t* mask, int T, const int* cu_seqlens, int n_seqs, int n_streams,
                const alch_stream* streams, long long capacity, int* kept_index, int* cu_kept,
                int* n_kept_and_status, void* workspace, hipStream_t stream, bool traced) {
    int* block_offsets = static_cast<int*>(workspace);
    const int nblocks = T > 0 ? ceil_div(T, kTokPerBlock) : 0;
    if (T <= kOneLaunchTokens) {
        TraceScope ts(traced ? kTracePackScan : kTraceRowOps, 0.0, (double)T + 4.0 * (n_seqs + 1), stream);
        const int chunk = (int)round_up((size_t)ceil_div(T > 0 ? T : 1, kOneLaunchThreads), kTokPerThread);
        k_pack_scan_one<<<1, kOneLaunchThreads, 0, stream>>>(mask, T, chunk, cu_seqlens, n_seqs + 1, kept_index, cu_kept,
                                                             n_kept_and_status, capacity);
    } else {
    TraceScope ts(traced ? kTracePackScan : kTraceRowOps, 0.0, (double)T + 4.0 * (n_seqs + 1), stream);
    if (nblocks > 0) k_pack_count<<<nblocks, kScanThreads, 0, stream>>>(mask, T, block_offsets);
    k_pack_scan_blocks<<<1, kScanThreads, 0, stream>>>(block_offsets, nblocks, n_kept_and_status, capacity);
    if (nblocks > 0) k_pack_fill<<<nblocks, kScanThreads, 0, stream>>>(mask, T, block_offsets, kept_index, capacity);
    k_pack_cu<<<n_seqs + 1, 64, 0, stream>>>(mask, cu_seqlens, n_seqs + 1, block_offsets, nblocks,
                                              n_kept_and_status, cu_kept);
    }
    ALCH_HIP_TRY(hipGetLastError());
    return launch_pack_gather(T, n_streams, streams, capacity, kept_index, n_kept_and_status, stream, traced);
}

// The gather alone, from an index and a row count already on the device.
int launch_pack_gather(int T, int n_streams, const alch_stream* streams, long long capacity, const int* kept_index,
                       const int* n_kept_and_status, hipStream_t stream, bool traced) {
    if (T == 0 || capacity == 0) return ALCH_OK;

    // traced bytes of the gather: per kept row (read once + written once); the row count is on the device
    double row_bytes_rw = 0;
    for (int k = 0; k < n_streams; ++k) row_bytes_rw += 2.0 * (double)streams[k].row_bytes;
    TraceScope ts(traced ? kTracePackGather : kTraceRowOps, 0.0, row_bytes_rw, stream);

    long long max_rows = (long long)T < capacity ? (long long)T : capacity;
    int grid = (int)(max_rows < (long long)kGatherGridMax ? max_rows : (long long)kGatherGridMax);
    for (int base = 0; base < n_streams; base += kMaxStreamsPerLaunch) {
        GatherArgs a;
        a.n = n_streams - base < kMaxStreamsPerLaunch ? n_streams - base : kMaxStreamsPerLaunch;
        bool vec16 = true;
        for (int k = 0; k < a.n; ++k) {
            const alch_stream& s = streams[base + k];
            a.src[k] = static_cast<const char*>(s.src);
            a.dst[k] = static_cast<char*>(s.dst);
            a.row_bytes[k] = s.row_bytes;
            a.src_stride[k] = s.src_row_stride_bytes;
            vec16 = vec16 && aligned16(s.src) && aligned16(s.dst) && s.row_bytes % 16 == 0 &&
                    s.src_row_stride_bytes % 16 == 0;
        }
        if (vec16)
            k_pack_gather<u32x4><<<grid, 256, 0, stream>>>(a, kept_index, n_kept_and_status, capacity);
        else
            k_pack_gather<unsigned int><<<grid, 256, 0, stream>>>(a, kept_index, n_kept_and_status, capacity);
    }
    ALCH_HIP_TRY(hipGetLastError());
    return ALCH_OK;
}

}  // namespace alch
