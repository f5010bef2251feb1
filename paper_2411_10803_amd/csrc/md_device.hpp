// Device-side building blocks shared by the three stages: bf16 storage helpers, 64-lane wavefront
// reductions, deterministic block reductions / scans and a block-wide radix select.
// Written for gfx950 (wave64) only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace md {

constexpr int kWave = 64;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
// wave index within the block, as a scalar (the compiler cannot see that threadIdx.x / 64 is wave-uniform)
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// v_exp_f32 / v_log_f32: base-2, about 1 ulp, results below 2^-126 flush to zero.  Used where the
// argument is a (score - max) difference, so neither overflow nor denormal results matter.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Cross-lane steps on the DPP path (one VALU instruction each, no LDS round trip).
// quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140:
// after the four steps every lane of a 16-lane row holds the row's result; the four rows are then
// combined in a fixed order from lanes 0, 16, 32, 48.
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF>
__device__ __forceinline__ int dpp_i(int old, int src) {
    return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, BANK_MASK, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v), __float_as_int(v))); }

__device__ __forceinline__ float lane_bcast_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f<0xB1>(v); v += dpp_f<0x4E>(v); v += dpp_f<0x141>(v); v += dpp_f<0x140>(v);
    return (lane_bcast_f(v, 0) + lane_bcast_f(v, 16)) + (lane_bcast_f(v, 32) + lane_bcast_f(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v)); v = fmaxf(v, dpp_f<0x4E>(v)); v = fmaxf(v, dpp_f<0x141>(v)); v = fmaxf(v, dpp_f<0x140>(v));
    return fmaxf(fmaxf(lane_bcast_f(v, 0), lane_bcast_f(v, 16)), fmaxf(lane_bcast_f(v, 32), lane_bcast_f(v, 48)));
}
__device__ __forceinline__ int wave_sum_i(int v) {
    v += dpp_i<0xB1>(v, v); v += dpp_i<0x4E>(v, v); v += dpp_i<0x141>(v, v); v += dpp_i<0x140>(v, v);
    return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
           (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, (uint32_t)dpp_i<0xB1>((int)v, (int)v)); v = min(v, (uint32_t)dpp_i<0x4E>((int)v, (int)v));
    v = min(v, (uint32_t)dpp_i<0x141>((int)v, (int)v)); v = min(v, (uint32_t)dpp_i<0x140>((int)v, (int)v));
    const uint32_t a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    const uint32_t c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return min(min(a, b), min(c, d));
}
// Sum over aligned groups of G consecutive lanes (G a power of two); every lane of a group gets the
// group's sum.  Up to 16 lanes this is pure DPP; wider groups finish with lane exchanges.
template <int G>
__device__ __forceinline__ float group_sum(float v) {
    if (G >= 2) v += dpp_f<0xB1>(v);
    if (G >= 4) v += dpp_f<0x4E>(v);
    if (G >= 8) v += dpp_f<0x141>(v);
    if (G >= 16) v += dpp_f<0x140>(v);
    if (G >= 32) v += __shfl_xor(v, 16, kWave);
    if (G >= 64) v += __shfl_xor(v, 32, kWave);
    return v;
}
__device__ __forceinline__ float group_sum_rt(float v, int g) {
    if (g >= 2) v += dpp_f<0xB1>(v);
    if (g >= 4) v += dpp_f<0x4E>(v);
    if (g >= 8) v += dpp_f<0x141>(v);
    if (g >= 16) v += dpp_f<0x140>(v);
    if (g >= 32) v += __shfl_xor(v, 16, kWave);
    if (g >= 64) v += __shfl_xor(v, 32, kWave);
    return v;
}

// 64-bit minimum: first the high words, then the low words of the lanes that hold the winning high word
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    const uint32_t mh = wave_min_u32(hi);
    const uint32_t ml = wave_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
    return ((uint64_t)mh << 32) | ml;
}
// Inclusive prefix sum over the 64 lanes: row_shr 1, 2, 4, 8 (0x111..0x118; lanes without a source
// add 0), then row_bcast15 into rows 1 and 3 and row_bcast31 into rows 2 and 3.
__device__ __forceinline__ int wave_incl_scan_i(int s) {
    s += dpp_i<0x111>(0, s); s += dpp_i<0x112>(0, s); s += dpp_i<0x114>(0, s); s += dpp_i<0x118>(0, s);
    s += dpp_i<0x142, 0xA>(0, s); s += dpp_i<0x143, 0xC>(0, s);
    return s;
}

// Block reductions: fixed tree (lanes by DPP steps, then the per-wave results -- one per lane --
// by the same steps) -> the result is the same on every run and on every thread.
// `red` holds >= blockDim.x/64 entries (at most 16 waves per block).
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    return wave_sum(lane_id() < nw ? red[lane_id()] : 0.f);
}
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    return wave_max(lane_id() < nw ? red[lane_id()] : -INFINITY);
}
__device__ __forceinline__ int block_sum_i(int v, int* red) {
    v = wave_sum_i(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    return wave_sum_i(lane_id() < nw ? red[lane_id()] : 0);
}

// Prefix of this wave among the per-wave totals in `red` (one LDS read per lane + a lane scan).
__device__ __forceinline__ int wave_prefix_of_totals(const int* red, int& total) {
    const int nw = blockDim.x >> 6, lane = lane_id(), w = wave_id();
    const int mine = lane < nw ? red[lane] : 0;
    const int incl = wave_incl_scan_i(mine);
    total = __builtin_amdgcn_readlane(incl, kWave - 1);
    return __builtin_amdgcn_readlane(incl, w) - __builtin_amdgcn_readlane(mine, w);
}

// Exclusive scan of a 0/1 flag over the block, in thread order.  Returns this thread's rank and
// the block total.  `red` holds >= blockDim.x/64 ints.
__device__ __forceinline__ int block_rank(bool flag, int* red, int& total) {
    const unsigned long long bal = __ballot(flag);
    const int lane = lane_id();
    const int below = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) red[wave_id()] = __popcll(bal);
    __syncthreads();
    return wave_prefix_of_totals(red, total) + below;
}

// Order-preserving composite key: larger score first, then smaller tie value first.
// `score` must be >= 0 (its bit pattern is then monotone); `tie` in [0, 2^31).
__device__ __forceinline__ uint64_t rank_key(float score, int tie) {
    return ((uint64_t)__float_as_uint(score) << 32) | (uint32_t)(0x7FFFFFFF - tie);
}

// Block-wide radix select: the k-th largest (k >= 1) of the distinct 64-bit keys produced by
// `key(i, ok)` for i in [0, n) (ok=false: item absent).  8-bit digits from the top; stops as
// soon as the chosen bin is taken whole.  Returns `bound` such that item i is among the k largest
// iff (key_i >> shift) >= bound.  If fewer than k items exist every item is selected.
// `hist` is 256 ints of shared memory.  All threads of the block must call it.
struct SelectBound { uint64_t bound; int shift; };

template <class KeyFn>
__device__ __forceinline__ SelectBound block_radix_select(KeyFn key, int n, int k, int* hist) {
    uint64_t prefix = 0;
    int shift = 64;
    __shared__ int s_digit, s_k, s_done;
    int kk = k;
    if (k <= 0) return SelectBound{~0ull, 0};               // nothing selected
    for (int pass = 0; pass < 8; ++pass) {
        const int sh = 56 - 8 * pass;
        __syncthreads();
        for (int i = threadIdx.x; i < 256; i += blockDim.x) hist[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            bool ok;
            const uint64_t kv = key(i, ok);
            if (ok && (pass == 0 || (kv >> shift) == prefix)) atomicAdd(&hist[(kv >> sh) & 0xFF], 1);
        }
        __syncthreads();
        if (threadIdx.x < kWave) {
            // digits 255..0 handled 4 per lane, high digits in low lanes
            const int lane = threadIdx.x;
            int c[4], s = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) { c[t] = hist[255 - (lane * 4 + t)]; s += c[t]; }
            const int incl = wave_incl_scan_i(s);           // inclusive scan over lanes
            int run = incl - s;                             // items in strictly higher digits
            const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
            if (lane == 0 && total < kk) { s_digit = 0; s_k = kk; s_done = 2; }   // fewer than k items
            if (total >= kk) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (run < kk && run + c[t] >= kk) {
                        s_digit = 255 - (lane * 4 + t);
                        s_k = kk - run;
                        s_done = (run + c[t] == kk) ? 1 : 0;
                    }
                    run += c[t];
                }
            }
        }
        __syncthreads();
        if (s_done == 2) return SelectBound{0ull, 63};      // select everything (keys < 2^63)
        prefix = (prefix << 8) | (uint64_t)s_digit;
        shift = sh;
        kk = s_k;
        if (s_done == 1) break;
    }
    return SelectBound{prefix, shift};
}

// Same selection with the keys held in registers (IPT per thread, 0 = absent; real keys are never 0
// as long as the tie value is below 2^31 - 1), built for a short chain of dependent steps:
//   - the scores of one sample share their leading bits (sign, most of the exponent): the block's
//     smallest and largest score are found first and the passes start below the bits they share, so
//     the first histogram is spread over its bins instead of piling onto two or three of them;
//   - three histograms take turns (pass p counts into hist[p % 3] and clears hist[(p + 1) % 3], which
//     nobody reads between the two barriers around it), and every wave scans the finished histogram
//     itself: one barrier per pass and no hand-over of the result through LDS.
// `hist`: 768 ints of shared memory whose first 256 the caller has zeroed, with a block barrier
// between the zeroing and this call.  All threads of the block (at most 16 waves) must call it.
constexpr int kSelectHistInts = 768;
template <int IPT>
__device__ __forceinline__ SelectBound block_select_topk(const uint64_t (&key)[IPT], int k, int* hist) {
    if (k <= 0) return SelectBound{~0ull, 0};               // nothing selected
    const int lane = lane_id(), wv = wave_id(), nw = blockDim.x >> 6;
    // leading bits common to every present key's score
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int t = 0; t < IPT; ++t)
        if (key[t] != 0) { lo = min(lo, (uint32_t)(key[t] >> 32)); hi = max(hi, (uint32_t)(key[t] >> 32)); }
    lo = wave_min_u32(lo);
    hi = ~wave_min_u32(~hi);
    if (lane == 0) { hist[512 + wv] = (int)lo; hist[528 + wv] = (int)hi; }     // hist[2] is not in use before pass 1
    __syncthreads();
    lo = wave_min_u32(lane < nw ? (uint32_t)hist[512 + lane] : 0xFFFFFFFFu);
    hi = ~wave_min_u32(lane < nw ? ~(uint32_t)hist[528 + lane] : 0xFFFFFFFFu);
    if (lo > hi) return SelectBound{0ull, 63};              // no key present: "select everything" selects nothing
    const int skip = lo == hi ? 32 : __clz((int)(lo ^ hi));
    int sh = 56 - skip, shift = 64 - skip;
    uint64_t prefix = skip > 0 ? ((uint64_t)hi << 32) >> shift : 0ull;
    int kk = k;
    bool first = skip == 0;
    for (int pass = 0;; ++pass) {
        int* h = hist + (pass % 3) * 256;
        int* hn = hist + ((pass + 1) % 3) * 256;
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const uint64_t kv = key[t];
            if (kv != 0 && (first || (kv >> shift) == prefix)) atomicAdd(&h[(kv >> sh) & 0xFF], 1);
        }
        if (threadIdx.x < 256) hn[threadIdx.x] = 0;
        __syncthreads();
        // digits 255..0, four per lane, high digits in low lanes; every wave does the same scan
        int c[4], s = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) { c[t] = h[255 - (lane * 4 + t)]; s += c[t]; }
        const int incl = wave_incl_scan_i(s);
        const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
        if (total < kk) return SelectBound{0ull, 63};       // fewer than k items: select everything (keys < 2^63)
        int run = incl - s;                                 // items in strictly higher digits
        const bool mine = run < kk && incl >= kk;           // the lane whose four digits hold the k-th item
        int packed = 0;
        if (mine) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (run < kk && run + c[t] >= kk)
                    packed = (255 - (lane * 4 + t)) | ((run + c[t] == kk ? 1 : 0) << 8) | ((kk - run) << 9);
                run += c[t];
            }
        }
        packed = __builtin_amdgcn_readlane(packed, __builtin_ctzll(__ballot(mine)));
        const int width = shift - sh;                       // 8, less when the last digit overlaps its predecessor
        prefix = (prefix << width) | ((uint64_t)(packed & 0xFF) & ((1ull << width) - 1ull));
        shift = sh;
        kk = packed >> 9;
        first = false;
        if (((packed >> 8) & 1) || sh == 0) break;          // the chosen bin is taken whole, or no bits are left
        sh = max(sh - 8, 0);
    }
    return SelectBound{prefix, shift};
}

// Block-wide minimum of 64-bit values (same result on every thread).  `red` holds >= blockDim.x/64 entries.
__device__ __forceinline__ uint64_t block_min_u64(uint64_t v, uint64_t* red) {
    v = wave_min_u64(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    return wave_min_u64(lane_id() < nw ? red[lane_id()] : ~0ull);
}

// Exclusive prefix sum over the block, in thread order.  Returns this thread's prefix; `total` =
// block sum.  `red` holds >= blockDim.x/64 ints.  Several small counters can share the word.
__device__ __forceinline__ int block_exscan_i(int v, int* red, int& total) {
    const int incl = wave_incl_scan_i(v);
    __syncthreads();
    if (lane_id() == kWave - 1) red[wave_id()] = incl;
    __syncthreads();
    return wave_prefix_of_totals(red, total) + incl - v;
}

}  // namespace md
