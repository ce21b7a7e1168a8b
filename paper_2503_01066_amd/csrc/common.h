// Internal helpers shared by the translation units of libalch (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "alch.h"

namespace alch {

// Records a formatted message for alch_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define ALCH_HIP_TRY(expr)                                                              \
    do {                                                                                \
        hipError_t e__ = (expr);                                                        \
        if (e__ != hipSuccess)                                                          \
            return ::alch::fail(ALCH_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

#define ALCH_TRY(expr)              \
    do {                            \
        int rc__ = (expr);          \
        if (rc__ != ALCH_OK) return rc__; \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
inline size_t dtype_size(alch_dtype d) { return d == ALCH_BF16 ? 2 : 4; }

// Bump allocator over the caller's workspace (256-byte aligned slices).
struct Arena {
    char* base;
    size_t size, used;
    Arena(void* p, size_t n) : base(static_cast<char*>(p)), size(n), used(0) {}
    void* take(size_t bytes) {
        size_t off = round_up(used, 256);
        used = off + bytes;
        return base ? base + off : nullptr;
    }
    bool ok() const { return used <= size; }
};

// Optional per-launch timing (alch_trace_enable): when on, a TraceScope brackets the kernels
// launched inside it with two HIP events on their stream.
enum TraceKind { kTraceGemmMfma = 0, kTraceGemmGeneric = 1, kTracePackScan = 2, kTracePackGather = 3,
                 kTraceAttnBwd = 4, kTraceAttnFwd = 5, kTraceRowOps = 6, kTraceCrossEntropy = 7, kTraceLora = 8 };
struct TraceScope {
    void* rec;
    hipStream_t stream;
    TraceScope(int kind, double flops, double bytes, hipStream_t s);
    ~TraceScope();
};

}  // namespace alch
