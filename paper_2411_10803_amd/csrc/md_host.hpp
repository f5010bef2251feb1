// Host-side helpers of the C ABI: thread-local error text, argument checks, workspace carving.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/mustdrop.h"

namespace md {

char* error_buffer();                       // thread-local, 512 bytes
int fail(int code, const char* fmt, ...);   // formats into the buffer, returns code
void clear_error();

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of the caller's workspace.  With base == nullptr it only
// measures (used by the *_workspace_bytes functions, so sizes and carving cannot drift apart).
struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base(static_cast<char*>(b)) {}
    template <class T>
    T* take(size_t count) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += round_up(count * sizeof(T), 256);
        return p;
    }
};

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MD_EHIP, "%s: %s", what, hipGetErrorString(e));
    return MD_OK;
}

inline size_t elt_size(int dtype) { return dtype == MD_BF16 ? 2 : 4; }

// Optional per-kernel timing (mustdrop_profile_start / _stop): when enabled, every launch is
// bracketed by a pair of HIP events on the launch stream.  Off by default: two branches per launch.
bool profiling();
// A pair of events for the next launch of `kernel_name` (timing session open), or two null handles.
void profile_events(const char* kernel_name, hipEvent_t* start, hipEvent_t* stop);

// Every kernel launch of the library.  In a timing session the launch carries an event pair that
// receives the dispatch's own begin and end timestamps (the figures a kernel trace shows), not the
// time at which a marker on the stream is reached.
#define MD_LAUNCH(name, st, kern, grid, block, shmem, ...)                                         \
    do {                                                                                           \
        if (md::profiling()) {                                                                     \
            hipEvent_t md_e0 = nullptr, md_e1 = nullptr;                                           \
            md::profile_events(name, &md_e0, &md_e1);                                              \
            hipExtLaunchKernelGGL(kern, dim3(grid), dim3(block), shmem, st, md_e0, md_e1, 0, __VA_ARGS__); \
        } else {                                                                                   \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(block), shmem, st, __VA_ARGS__);              \
        }                                                                                          \
    } while (0)

}  // namespace md
