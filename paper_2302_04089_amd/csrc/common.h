// Internal helpers shared by the translation units of libziplm (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "ziplm.h"

#define ZIPLM_HIP_TRY(expr)                                   \
    do {                                                      \
        hipError_t _e = (expr);                               \
        if (_e != hipSuccess) return ZIPLM_ERR_DEVICE;        \
    } while (0)

namespace ziplm {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of a caller-provided workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t count) {
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += align_up(count * sizeof(T));
        return p;
    }
};

// Zero-fills `bytes` bytes (a multiple of 16, 16-byte aligned) with a small kernel on `stream`.  Used instead of
// hipMemsetAsync for the library's flags and counters: a fill kernel is an ordinary graph node if the caller
// captures the stream, a memset node is not always replayed correctly.
int zero_fill(void *p, size_t bytes, hipStream_t stream);

inline bool workspace_ok(const void *ws, size_t have, size_t need) {
    if (need == 0) return true;
    return ws != nullptr && (reinterpret_cast<uintptr_t>(ws) % kAlign) == 0 && have >= need;
}

}  // namespace ziplm
