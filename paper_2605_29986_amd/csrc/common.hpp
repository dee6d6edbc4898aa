// Shared host-side helpers of the CFGzip HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cfgzip.h"

namespace cfgzip {

constexpr int kWave = 64;  // CDNA wavefront width

// Per-host-thread record of the last failing HIP status.
void set_last_hip_error(hipError_t e);

inline int check_hip(hipError_t e) {
    if (e == hipSuccess) return CFGZIP_OK;
    set_last_hip_error(e);
    return CFGZIP_E_HIP;
}

// Launch errors surface through hipGetLastError right after the launch.
inline int check_launch() { return check_hip(hipGetLastError()); }

#define CFGZIP_TRY(expr)                         \
    do {                                         \
        int cfgzip_rc_ = (expr);                 \
        if (cfgzip_rc_ != CFGZIP_OK) return cfgzip_rc_; \
    } while (0)

inline int64_t words_for(int64_t n) { return (n + 31) / 32; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Carves consecutive 256-byte aligned regions out of a caller-provided workspace.
struct Carver {
    char *base;
    size_t used = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t count) {
        size_t off = used;
        used = align_up(used + count * sizeof(T), 256);
        return base ? reinterpret_cast<T *>(base + off) : nullptr;
    }
};

}  // namespace cfgzip
