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

// Element strides of a [B, tokens, H, d] tensor as the kernels take them (d elements contiguous).
struct KvLayout {
    long batch, token, head;
};

inline KvLayout dense_layout(long tokens, int H, int d) { return KvLayout{tokens * H * d, (long)H * d, (long)d}; }

inline bool is_dense(const KvLayout& l, long tokens, int H, int d) {
    return l.head == d && l.token == (long)H * d && l.batch == tokens * H * d;
}

// Bytes from the base pointer to the end of the last element.
inline size_t layout_extent_bytes(const KvLayout& l, int B, long tokens, int H, int d) {
    return (size_t)((B - 1) * l.batch + (tokens - 1) * l.token + (H - 1) * l.head + d) * 2;
}

// Reads a caller's layout (NULL = dense token-major) and checks it: positive multiples of 8
// elements, axes nested without overlap.  Returns MD_OK or fails with MD_EINVAL / MD_ESHAPE.
inline int read_layout(const char* who, const char* what, const md_kv_layout* in, int B, long tokens, int H, int d,
                       KvLayout* out) {
    if (!in) { *out = dense_layout(tokens, H, d); return MD_OK; }
    const long s[3] = {(long)in->batch, (long)in->token, (long)in->head};
    const long n[3] = {(long)B, tokens, (long)H};
    for (int a = 0; a < 3; ++a) {
        if (s[a] <= 0 || s[a] % 8) return fail(MD_EINVAL, "%s: %s strides must be positive multiples of 8 elements", who, what);
        if (s[a] > (1l << 40)) return fail(MD_EINVAL, "%s: %s stride too large", who, what);
    }
    int ord[3] = {0, 1, 2};                                   // axes by ascending stride (extent-1 axes first on ties)
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (s[ord[j]] < s[ord[i]] || (s[ord[j]] == s[ord[i]] && n[ord[j]] < n[ord[i]])) { int t = ord[i]; ord[i] = ord[j]; ord[j] = t; }
    long need = d;                                            // smallest stride an axis may have so far
    for (int i = 0; i < 3; ++i) {
        const int a = ord[i];
        if (n[a] > 1 && s[a] < need) return fail(MD_ESHAPE, "%s: %s layout overlaps itself (stride %ld < %ld)", who, what, s[a], need);
        if (n[a] > 1) need = s[a] * n[a];
    }
    *out = KvLayout{s[0], s[1], s[2]};
    return MD_OK;
}

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
