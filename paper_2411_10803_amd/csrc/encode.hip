// Stage 1 -- vision encoding (Sec. 3.3): Key Retaining (Eq. 6-7, budget form) and Local Spatial
// Merging (Eq. 5), followed by stable compaction of the survivors.
//
// Launch plan (all on the caller's stream, no host synchronisation):
//   encode_scores_kernel one launch, two kinds of waves:
//       window waves     one wave per window: Gram matrix in registers -> S    (HBM: reads x once)
//       key-row waves    one wave per four key rows: q_cls . k_j per head      (HBM: reads k_cls once)
//   encode_decide_kernel one block per sample: softmax + head mean, radix top-k -> O, merge
//                        decisions, prefix sum of survivors, small outputs    (tiny)
//   encode_emit_kernel  one wave per window: row copies / mass-weighted means (re-reads x, writes out_x)
#include "md_device.hpp"
#include "md_host.hpp"

#include <mutex>

namespace md {
namespace {

constexpr float kLog2eE = 1.4426950408889634f;
constexpr int kMaxWindow = 16;                   // = the length of EncodeDims::moff
#ifndef MD_ENC_WAVES
#define MD_ENC_WAVES 4
#endif
constexpr int kEncWaves = MD_ENC_WAVES;          // waves (= work items) per block of the wave-per-item kernels
constexpr int kMaxClsHeads = 256;

struct EncodeDims {
    int B, T, Hg, Wg, D, Hc, dc;
    int kt, kh, kw;
    int M, W, ws, nwx, nwy, nwt;
    int clipped;      // the window does not divide the grid: windows at the far border hold fewer tokens
    int moff[16];     // member_offset(m), m < ws: filled by the host so that kernels get them as scalars
};

// Token of member m of window w; -1 for a member that a clipped border window does not have.
__device__ __forceinline__ int member_token(const EncodeDims& p, int w, int m) {
    const int wx = w % p.nwx, wy = (w / p.nwx) % p.nwy, wt = w / (p.nwx * p.nwy);
    const int dx = m % p.kw, dy = (m / p.kw) % p.kh, dt = m / (p.kw * p.kh);
    const int t = wt * p.kt + dt, y = wy * p.kh + dy, x = wx * p.kw + dx;
    if (p.clipped && (t >= p.T || y >= p.Hg || x >= p.Wg)) return -1;
    return (t * p.Hg + y) * p.Wg + x;
}
__device__ __forceinline__ bool member_in_grid(const EncodeDims& p, int w, int m) {
    return !p.clipped || member_token(p, w, m) >= 0;
}
// member_token(p, w, m) = window_base(p, w) + member_offset(p, m)
__device__ __forceinline__ int window_base(const EncodeDims& p, int w) {
    const int wx = w % p.nwx, wy = (w / p.nwx) % p.nwy, wt = w / (p.nwx * p.nwy);
    return (wt * p.kt * p.Hg + wy * p.kh) * p.Wg + wx * p.kw;
}
__host__ __device__ __forceinline__ int member_offset(const EncodeDims& p, int m) {
    const int dx = m % p.kw, dy = (m / p.kw) % p.kh, dt = m / (p.kw * p.kh);
    return (dt * p.Hg + dy) * p.Wg + dx;
}
// A wave that works on one window: lane m < ws computes member m's token (one division sequence
// for all members instead of one per member); read back with wave_member().
__device__ __forceinline__ int lane_member_token(const EncodeDims& p, int w, int lane) {
    return lane < p.ws ? member_token(p, w, lane) : 0;
}
__device__ __forceinline__ int wave_member(int per_lane, int m) { return __builtin_amdgcn_readlane(per_lane, m); }

__device__ __forceinline__ int window_of_token(const EncodeDims& p, int tok) {
    const int x = tok % p.Wg, y = (tok / p.Wg) % p.Hg, t = tok / (p.Wg * p.Hg);
    return ((t / p.kt) * p.nwy + (y / p.kh)) * p.nwx + (x / p.kw);
}

// One 16-byte vector of a row, widened to fp32.  VEC = 4 (fp32) or 8 (bf16).
template <bool BF> struct Vec;
template <> struct Vec<false> {
    static constexpr int N = 4;
    // a vector as loaded, and the dot product of two of them added to acc (elements in ascending order)
    using Raw = f32x4;
    __device__ static __forceinline__ Raw load_raw(const void* row, int c) { return *reinterpret_cast<const f32x4*>(static_cast<const float*>(row) + c); }
    __device__ static __forceinline__ Raw load_raw_once(const void* row, int c) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<const float*>(row) + c)); }
    __device__ static __forceinline__ Raw zero() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ static __forceinline__ float dot(const Raw& a, const Raw& b, float acc) {
        acc = fmaf(a.x, b.x, acc); acc = fmaf(a.y, b.y, acc); acc = fmaf(a.z, b.z, acc); return fmaf(a.w, b.w, acc);
    }
    __device__ static __forceinline__ void load(const void* row, int c, float (&o)[4]) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(static_cast<const float*>(row) + c);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    // data that is not read again: streaming load
    __device__ static __forceinline__ void load_once(const void* row, int c, float (&o)[4]) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<const float*>(row) + c));
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    __device__ static __forceinline__ void store(void* row, int c, const float (&o)[4]) {
        f32x4 v; v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3];
        *reinterpret_cast<f32x4*>(static_cast<float*>(row) + c) = v;
    }
};
template <> struct Vec<true> {
    static constexpr int N = 8;
    // bf16 pairs stay packed: v_dot2c_f32_bf16 multiplies two pairs and adds both products to an fp32
    // accumulator (the products of bf16 values are exact in fp32), one instruction per two elements and
    // no widening
    using Raw = u32x4;
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    __device__ static __forceinline__ Raw load_raw(const void* row, int c) { return *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(row) + c); }
    __device__ static __forceinline__ Raw load_raw_once(const void* row, int c) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(row) + c)); }
    __device__ static __forceinline__ Raw zero() { return u32x4{0u, 0u, 0u, 0u}; }
    __device__ static __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
    }
    __device__ static __forceinline__ float dot(const Raw& a, const Raw& b, float acc) {
        acc = dot2(a.x, b.x, acc); acc = dot2(a.y, b.y, acc); acc = dot2(a.z, b.z, acc); return dot2(a.w, b.w, acc);
    }
    __device__ static __forceinline__ void widen(const u32x4 v, float (&o)[8]) {
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ void load(const void* row, int c, float (&o)[8]) {
        widen(*reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(row) + c), o);
    }
    __device__ static __forceinline__ void load_once(const void* row, int c, float (&o)[8]) {
        widen(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(row) + c)), o);
    }
    __device__ static __forceinline__ void store(void* row, int c, const float (&o)[8]) {
        u32x4 v;
        v.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
        v.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
        v.z = f32_to_bf16(o[4]) | (f32_to_bf16(o[5]) << 16);
        v.w = f32_to_bf16(o[6]) | (f32_to_bf16(o[7]) << 16);
        *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(row) + c) = v;
    }
};

// ---------------------------------------------------------------------------------------------
// Eq. 6, the part that needs no global view.  With x[h][j] = log2(e) * q_cls[b][h] . k_cls[b][j][h] / sqrt(dc),
// j = 0..M, one wave takes kClsRows consecutive key rows of a sample (their loads are in flight
// together) and leaves, per head h and for its group g of rows,
//     part[b][h][g] = (m, z):  m = max of x over the rows that count (the CLS row and the valid tokens),
//                              z = sum of exp2(x - m) over them,
//     num[b][j][h]  = exp2(x[h][j] - m)   for each of those rows (heads contiguous),
// so that the decision kernel gets a probability as num * exp2(m - m_h) / Z_h with one factor per
// (head, group): no exponential per (head, token) on the one CU that decides for a sample.
// A head covers vph = dc/VEC consecutive 16-byte vectors (a power of two), so the per-head sums are
// segmented butterflies over vph lanes (or whole-wave sums if vph >= 64).
constexpr int kClsRows = 8;
__host__ __device__ __forceinline__ int cls_groups(int M) { return (M + 1 + kClsRows - 1) / kClsRows; }

template <bool BF>
__device__ __forceinline__ void cls_logits_rows(
    long item, const void* __restrict__ q_cls, const void* __restrict__ k_cls, const uint8_t* __restrict__ valid,
    const EncodeDims& p, float* __restrict__ logits, float2* __restrict__ part)
{
    constexpr int VEC = Vec<BF>::N;
    constexpr int R = kClsRows;
    const int lane = lane_id();
    const int gps = cls_groups(p.M);
    if (item >= (long)p.B * gps) return;
    const int b = (int)(item / gps), g = (int)(item % gps), j0 = g * R;
    // wave-uniform.  Loads are never guarded one by one (a guarded load waits for the one before it):
    // addresses are clamped into the sample instead and what was read for an inactive row is ignored.
    bool act[R];
    uint32_t vbyte[R];
#pragma unroll
    for (int r = 0; r < R; ++r) vbyte[r] = valid ? valid[(size_t)b * p.M + min(max(j0 + r - 1, 0), p.M - 1)] : 1u;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int j = j0 + r;
        act[r] = j <= p.M && (j == 0 || vbyte[r] != 0);
    }

    const size_t esz = BF ? 2 : 4;
    const char* qrow = static_cast<const char*>(q_cls) + (size_t)b * p.D * esz;
    const size_t rowb = (size_t)p.D * esz;
    const char* kb0 = static_cast<const char*>(k_cls) + (size_t)b * (p.M + 1) * rowb;
    const char* krow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) krow[r] = kb0 + (size_t)min(j0 + r, p.M) * rowb;
    const int nvec = p.D / VEC, vph = p.dc / VEC;
    const float scale = 1.0f / sqrtf((float)p.dc);
    float* out = logits + ((size_t)b * (p.M + 1) + j0) * p.Hc;
    float2* pout = part + (size_t)b * p.Hc * gps + g;
    // the R logits of one head -> numerators (in place) and their statistics (every lane that holds
    // them computes the same values)
    auto finish = [&](float (&lg)[R]) -> float2 {
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (act[r]) mx = fmaxf(mx, lg[r] * kLog2eE);
        float z = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            lg[r] = act[r] ? fast_exp2(fmaf(lg[r], kLog2eE, -mx)) : 0.f;
            z += lg[r];
        }
        return make_float2(mx, z);
    };

    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    const int iters = (nvec + kWave - 1) / kWave;
    for (int it = 0; it < iters; ++it) {
        const int idx = it * kWave + lane;
        float part_r[R];
#pragma unroll
        for (int r = 0; r < R; ++r) part_r[r] = 0.f;
        {
            const int ic = min(idx, nvec - 1);       // lanes beyond the row repeat its last vector and drop it
            typename Vec<BF>::Raw kv[R];
            const typename Vec<BF>::Raw qv = Vec<BF>::load_raw(qrow, ic * VEC);
#pragma unroll
            // the key rows are read exactly once: streaming loads, so that they do not push x (read again by
            // the emit kernel) out of the Infinity Cache
            for (int r = 0; r < R; ++r) kv[r] = Vec<BF>::load_raw_once(krow[r], ic * VEC);
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (act[r] && idx < nvec) part_r[r] = Vec<BF>::dot(qv, kv[r], part_r[r]);
        }
        if (vph < kWave) {
            float lg[R];
#pragma unroll
            for (int r = 0; r < R; ++r) lg[r] = group_sum_rt(part_r[r], vph) * scale;
            if (idx < nvec && (lane & (vph - 1)) == 0) {
                const int h = idx / vph;
                pout[(size_t)h * gps] = finish(lg);
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if (act[r]) out[(size_t)r * p.Hc + h] = lg[r];
            }
        } else {
            const int per_head = vph / kWave;                 // iterations per head
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] += part_r[r];
            if ((it + 1) % per_head == 0) {
                float lg[R];
#pragma unroll
                for (int r = 0; r < R; ++r) { lg[r] = wave_sum(acc[r]) * scale; acc[r] = 0.f; }
                if (lane == 0) {
                    const int h = it / per_head;
                    pout[(size_t)h * gps] = finish(lg);
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        if (act[r]) out[(size_t)r * p.Hc + h] = lg[r];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 5: S_w = mean over unordered pairs of valid members of cos(x_m, x_n).  One wave per window;
// each lane owns a strided slice of the feature dimension and keeps the upper triangle of the
// Gram matrix (norms on the diagonal) in registers; one butterfly per entry at the end.
template <int WSM, bool BF>
__device__ __forceinline__ void window_sim_item(
    long item, const void* __restrict__ x, const uint8_t* __restrict__ valid, const EncodeDims& p, float* __restrict__ sim)
{
    constexpr int VEC = Vec<BF>::N;
    const int lane = lane_id();
    if (item >= (long)p.B * p.W) return;
    const int b = (int)(item / p.W), w = (int)(item % p.W);
    const size_t esz = BF ? 2 : 4;

    const char* rows[WSM];
    bool ok[WSM];
    const int tok_l = lane_member_token(p, w, lane);
    const int ok_l = lane < p.ws && tok_l >= 0 && (!valid || valid[(size_t)b * p.M + max(tok_l, 0)]);
#pragma unroll
    for (int m = 0; m < WSM; ++m) {
        // every slot gets a readable row (members beyond the window repeat member 0, invalid members
        // keep their own row): the loads below are unconditional and what they return is zeroed
        const int mm = m < p.ws ? m : 0;
        ok[m] = m < p.ws && wave_member(ok_l, mm) != 0;
        rows[m] = static_cast<const char*>(x) + ((size_t)b * p.M + max(wave_member(tok_l, mm), 0)) * p.D * esz;
    }
    float G[WSM * (WSM + 1) / 2];
#pragma unroll
    for (int i = 0; i < WSM * (WSM + 1) / 2; ++i) G[i] = 0.f;

    // small windows take two slices of the feature dimension per round (2*WSM loads in flight)
    constexpr int NS = WSM <= 4 ? 2 : 1;
    for (int c0 = lane * VEC; c0 < p.D; c0 += NS * kWave * VEC) {
        typename Vec<BF>::Raw v[NS][WSM];
        bool in[NS];
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            const int c = c0 + q * kWave * VEC;
            in[q] = c < p.D;
#pragma unroll
            for (int m = 0; m < WSM; ++m) v[q][m] = Vec<BF>::load_raw(rows[m], in[q] ? c : c0);
        }
#pragma unroll
        for (int q = 0; q < NS; ++q)
#pragma unroll
            for (int m = 0; m < WSM; ++m)
                if (!ok[m] || !in[q]) v[q][m] = Vec<BF>::zero();
#pragma unroll
        for (int q = 0; q < NS; ++q) {
            int idx = 0;
#pragma unroll
            for (int m = 0; m < WSM; ++m)
#pragma unroll
                for (int n = m; n < WSM; ++n) {
                    G[idx] = Vec<BF>::dot(v[q][m], v[q][n], G[idx]);
                    ++idx;
                }
        }
    }
#pragma unroll
    for (int i = 0; i < WSM * (WSM + 1) / 2; ++i) G[i] = wave_sum(G[i]);

    if (lane == 0) {
        float S = 0.f;
        int npairs = 0;
        float diag[WSM];
        {
            int idx = 0;
#pragma unroll
            for (int m = 0; m < WSM; ++m) { diag[m] = G[idx]; idx += WSM - m; }
        }
        int idx = 0;
#pragma unroll
        for (int m = 0; m < WSM; ++m)
#pragma unroll
            for (int n = m; n < WSM; ++n) {
                if (n > m && ok[m] && ok[n]) {
                    const float den = sqrtf(diag[m]) * sqrtf(diag[n]);
                    S += (diag[m] > 0.f && diag[n] > 0.f) ? G[idx] / den : 0.f;
                    ++npairs;
                }
                ++idx;
            }
        sim[(size_t)b * p.W + w] = npairs > 0 ? S / (float)npairs : 0.f;
    }
}

// One launch for both bandwidth-bound score passes: waves [0, B*W) take a window each (Eq. 5), the
// following waves a few key rows each (Eq. 6 logits; none when no key set is asked for).
template <int WSM, bool XBF, bool QKBF>
__global__ __launch_bounds__(256) void encode_scores_kernel(
    const void* __restrict__ x, const void* __restrict__ q_cls, const void* __restrict__ k_cls,
    const uint8_t* __restrict__ valid, EncodeDims p, int with_cls, float* __restrict__ sim, float* __restrict__ logits,
    float2* __restrict__ cls_part)
{
    const long item = (long)blockIdx.x * (blockDim.x >> 6) + wave_id();
    const long n_win = (long)p.B * p.W;
    if (item < n_win) window_sim_item<WSM, XBF>(item, x, valid, p, sim);
    else if (with_cls) cls_logits_rows<QKBF>(item - n_win, q_cls, k_cls, valid, p, logits, cls_part);
}

// ---------------------------------------------------------------------------------------------
// Per-sample decisions.  One block per sample.
__global__ __launch_bounds__(1024) void encode_decide_kernel(
    EncodeDims p, const uint8_t* __restrict__ valid, const float* __restrict__ mass_in,
    const float* __restrict__ logits, const float2* __restrict__ cls_part, const float* __restrict__ sim, float tau,
    int key_budget, int key_adaptive, float key_lambda, int32_t* __restrict__ key_count,
    float* __restrict__ acls, uint8_t* __restrict__ iskey, uint8_t* __restrict__ wmerged,
    int32_t* __restrict__ dstpos,
    int32_t* __restrict__ out_index, float* __restrict__ out_mass, uint8_t* __restrict__ out_is_key,
    uint8_t* __restrict__ out_valid, int32_t* __restrict__ out_count, int32_t* __restrict__ key_index,
    float* __restrict__ a_cls_out, float* __restrict__ window_sim_out)
{
    __shared__ float s_max[kMaxClsHeads], s_inv[kMaxClsHeads];
    __shared__ int s_hist[256];
    __shared__ int s_red[16];
    __shared__ float s_redf[16];
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wv = wave_id(), nw = blockDim.x >> 6;
    const int M = p.M, W = p.W;
    const uint8_t* vb = valid ? valid + (size_t)b * M : nullptr;
    const float* mb = mass_in ? mass_in + (size_t)b * M : nullptr;
    float* acls_b = acls + (size_t)b * M;
    uint8_t* iskey_b = iskey + (size_t)b * M;
    uint8_t* wm_b = wmerged + (size_t)b * W;
    int32_t* dst_b = dstpos + (size_t)b * M;

    // ---- Key Retaining
    if (key_budget > 0 || key_adaptive) {
        const float* lg = logits + (size_t)b * (M + 1) * p.Hc;       // numerators [row][head], see cls_logits_rows
        const int gps = cls_groups(M);
        const float2* pb = cls_part + (size_t)b * p.Hc * gps;
        for (int h = wv; h < p.Hc; h += nw) {
            const float2* pp = pb + (size_t)h * gps;
            float mx = -INFINITY;
            for (int g = lane; g < gps; g += kWave) mx = fmaxf(mx, pp[g].x);
            mx = wave_max(mx);
            float z = 0.f;
            for (int g = lane; g < gps; g += kWave) {
                const float2 v = pp[g];
                if (v.x > -INFINITY) z = fmaf(v.y, fast_exp2(v.x - mx), z);
            }
            z = wave_sum(z);
            if (lane == 0) { s_max[h] = mx; s_inv[h] = 1.0f / (z * (float)p.Hc); }
        }
        __syncthreads();
        for (int j = tid; j < M; j += blockDim.x) {
            float a = -INFINITY;
            if (!vb || vb[j]) {
                a = 0.f;
                const int g = (j + 1) / kClsRows;
                for (int h = 0; h < p.Hc; ++h)
                    a = fmaf(lg[(size_t)(j + 1) * p.Hc + h], fast_exp2(pb[(size_t)h * gps + g].x - s_max[h]) * s_inv[h], a);
            }
            acls_b[j] = a;
            if (a_cls_out) a_cls_out[(size_t)b * M + j] = a;
        }
        __syncthreads();
        auto keyfn = [&](int i, bool& ok) -> uint64_t {
            ok = !vb || vb[i];
            return ok ? rank_key(acls_b[i], i) : 0ull;
        };
        SelectBound sb{0ull, 63};
        float mu = 0.f;
        if (!key_adaptive) {                         // Eq. 7, budget form
            sb = block_radix_select(keyfn, M, key_budget, s_hist);
        } else {                                     // Eq. 7 as printed: a_cls > mu, mu = mean + lambda * std
            float s1 = 0.f;
            int cnt = 0;
            for (int j = tid; j < M; j += blockDim.x)
                if (!vb || vb[j]) { s1 += acls_b[j]; ++cnt; }
            s1 = block_sum(s1, s_redf);
            cnt = block_sum_i(cnt, s_red);
            const float mean = cnt > 0 ? s1 / (float)cnt : 0.f;
            float s2 = 0.f;
            for (int j = tid; j < M; j += blockDim.x)
                if (!vb || vb[j]) { const float dlt = acls_b[j] - mean; s2 = fmaf(dlt, dlt, s2); }
            s2 = block_sum(s2, s_redf);
            mu = mean + key_lambda * sqrtf(cnt > 0 ? s2 / (float)cnt : 0.f);
        }
        int running = 0;                             // keys so far; key_budget is the capacity of key_index
        for (int base = 0; base < M; base += blockDim.x) {
            const int j = base + tid;
            bool sel = false;
            if (j < M && (!vb || vb[j]))
                sel = key_adaptive ? acls_b[j] > mu : (rank_key(acls_b[j], j) >> sb.shift) >= sb.bound;
            if (j < M) iskey_b[j] = sel;
            int total;
            const int r = block_rank(sel, s_red, total);
            if (sel && running + r < key_budget) key_index[(size_t)b * key_budget + running + r] = j;
            running += total;
        }
        for (int r = running + tid; r < key_budget; r += blockDim.x) key_index[(size_t)b * key_budget + r] = -1;
        if (key_count && tid == 0) key_count[b] = running;
    } else {
        for (int j = tid; j < M; j += blockDim.x) {
            iskey_b[j] = 0;
            if (a_cls_out) a_cls_out[(size_t)b * M + j] = 0.f;
        }
    }
    __syncthreads();

    // ---- merge decision per window: S > tau, >= 2 valid members, no key member
    for (int w = tid; w < W; w += blockDim.x) {
        int n = 0;
        bool has_key = false;
        for (int m = 0; m < p.ws; ++m) {
            const int tok = member_token(p, w, m);
            if (tok < 0 || (vb && !vb[tok])) continue;
            ++n;
            has_key |= iskey_b[tok] != 0;
        }
        const float S = sim[(size_t)b * W + w];
        wm_b[w] = (n >= 2 && !has_key && S > tau) ? 1 : 0;
        if (window_sim_out) window_sim_out[(size_t)b * W + w] = S;
    }
    __syncthreads();

    // ---- survivors in ascending token index: exclusive prefix sum of the survivor flags
    int running = 0;
    for (int base = 0; base < M; base += blockDim.x) {
        const int j = base + tid;
        bool surv = false, merged = false;
        float mass = 0.f;
        if (j < M && (!vb || vb[j])) {
            const int w = window_of_token(p, j);
            merged = wm_b[w] != 0;
            if (!merged) {
                surv = true;
                mass = mb ? mb[j] : 1.0f;
            } else {
                int first = -1;
                for (int m = 0; m < p.ws; ++m) {
                    const int tok = member_token(p, w, m);
                    if (tok < 0 || (vb && !vb[tok])) continue;
                    if (first < 0) first = tok;
                    mass += mb ? mb[tok] : 1.0f;
                }
                surv = (first == j);
            }
        }
        int total;
        const int r = block_rank(surv, s_red, total);
        if (j < M) dst_b[j] = surv ? running + r : -1;
        if (surv) {
            const size_t o = (size_t)b * M + running + r;
            out_index[o] = j;
            out_mass[o] = mass;
            out_is_key[o] = merged ? 0 : iskey_b[j];
        }
        running += total;
    }
    if (tid == 0) out_count[b] = running;
    if (out_valid)
        for (int s = tid; s < M; s += blockDim.x) out_valid[(size_t)b * M + s] = s < running;
}

// ---------------------------------------------------------------------------------------------
// The same decisions for M <= 1024*IPT with a sample's tokens in registers (thread t owns the IPT
// consecutive tokens t*IPT ..): the kernel is a chain of dependent steps on one CU per sample, so it
// is built to be short rather than wide.
//   - the softmax denominators come from the per-wave statistics the score kernel left (a few
//     hundred pairs per head), while the own tokens' logits are already on their way;
//   - the top-k radix select starts below the bits that all scores share;
//   - key ranks and survivor ranks come from ONE block scan of a packed pair of counts.
#ifdef MD_DECIDE_TICKS
#define MD_DTICK(k) do { if (threadIdx.x == 0 && blockIdx.x == 0) ticks[k] = __builtin_readcyclecounter(); } while (0)
#else
#define MD_DTICK(k) do { } while (0)
#endif
template <int IPT, int WS>
__global__ __launch_bounds__(1024) void encode_decide_fast_kernel(
    EncodeDims p, const uint8_t* __restrict__ valid, const float* __restrict__ mass_in,
    const float* __restrict__ logits, const float2* __restrict__ cls_part, const float* __restrict__ sim,
    float tau, int key_budget, int key_adaptive, float key_lambda, int32_t* __restrict__ key_count,
    uint8_t* __restrict__ wmerged, int32_t* __restrict__ dstpos,
    int32_t* __restrict__ out_index, float* __restrict__ out_mass, uint8_t* __restrict__ out_is_key,
    uint8_t* __restrict__ out_valid, int32_t* __restrict__ out_count, int32_t* __restrict__ key_index,
    float* __restrict__ a_cls_out, float* __restrict__ window_sim_out)
{
    // [M] merged-window mass / scores (float), then [M] key flags and [M] token states, which take the place of
    // the [groups][16] factors of Eq. 6 (see decide_fast_lds_bytes)
    extern __shared__ __attribute__((aligned(16))) uint8_t s_dyn[];
    __shared__ int s_hist[kSelectHistInts];
    __shared__ int s_red[16];
    __shared__ float s_redf[16];
#ifdef MD_DECIDE_TICKS
    __shared__ long long ticks[12];
#endif
    MD_DTICK(0);
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const int M = p.M, W = p.W;
    if (tid < 256) s_hist[tid] = 0;                         // for block_select_topk, after later barriers
    float* s_tmass = reinterpret_cast<float*>(s_dyn);
    uint8_t* s_key = s_dyn + 4 * (size_t)M;
    uint8_t* s_state = s_key + M;                    // 0: not in a merged window, 1: first valid member, 2: merged away
    const uint8_t* vb = valid ? valid + (size_t)b * M : nullptr;
    const float* mb = mass_in ? mass_in + (size_t)b * M : nullptr;
    const int j0 = tid * IPT;                        // first own token (and first own window)
    const bool with_keys = key_budget > 0 || key_adaptive;
    const float* lg = logits + (size_t)b * (M + 1) * p.Hc;           // numerators [row][head], row 0 = CLS

    // ---- everything that depends on nothing is requested first (clamped or range-checked addresses, no
    // guarded loads: a guarded load would wait for the one before it)
    // Eq. 6: wave h owns head h (Hc <= 16 = waves of the block; waves beyond Hc contribute zeros).  Its
    // lanes take the head's per-group statistics (group = kClsRows rows, see cls_logits_rows).
    constexpr int PRE = 16;                          // heads
    constexpr int NPB = 2 * IPT + 1;                 // groups per lane: 64 * NPB >= cls_groups(1024 * IPT)
    constexpr bool EARLY = IPT <= 4;                 // registers allow the first batch to be requested up front
    const int gps = cls_groups(M);
    float2 pv[NPB];
    if (with_keys) {
        const float2* pp = cls_part + ((size_t)b * p.Hc + min(wv, p.Hc - 1)) * gps;
#pragma unroll
        for (int u = 0; u < NPB; ++u) pv[u] = pp[min(lane + u * kWave, gps - 1)];
    }
    // Numerators of the tokens tid + 1024*t: the 16 heads of a token are 64 consecutive bytes, four
    // 16-byte buffer loads (the token's offset in a vector register, the quarter's and the batch's in the
    // instruction and a scalar; tokens beyond M and heads beyond Hc fall outside the buffer's range and
    // read as zero).  The scores change hands through LDS afterwards.
    constexpr int PT = IPT < 4 ? IPT : 4;            // tokens per batch
    const int nrec = M * p.Hc * 4;
    const __amdgpu_buffer_rsrc_t rnum = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lg + p.Hc), 0, nrec, 0x00020000);
    f32x4 xl[PT][4];
    auto request_numerators = [&](int t0) {
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                xl[t][q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                    rnum, 4 * q < p.Hc ? tid * p.Hc * 4 + 16 * q : nrec, (t0 + t) * 1024 * p.Hc * 4, 0));
    };
    bool ok[IPT];
    float mass[IPT], simv[IPT];
    {
        uint32_t vbyte[IPT];
#pragma unroll
        for (int t = 0; t < IPT; ++t) vbyte[t] = vb ? vb[min(j0 + t, M - 1)] : 1u;
#pragma unroll
        for (int t = 0; t < IPT; ++t) mass[t] = mb ? mb[min(j0 + t, M - 1)] : 1.0f;
#pragma unroll
        for (int t = 0; t < IPT; ++t) simv[t] = sim[(size_t)b * W + min(tid + 1024 * t, W - 1)];
        if (EARLY && with_keys) request_numerators(0);
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const int j = j0 + t;
            ok[t] = j < M && vbyte[t] != 0;
            if (j >= M) mass[t] = 1.0f;
        }
    }
    bool sel[IPT];
#pragma unroll
    for (int t = 0; t < IPT; ++t) sel[t] = false;
    // What a window's decision needs besides the key flags, worked out while the loads above are on
    // their way: its first token, which members are valid, their count, first one and total mass.
    struct WinInfo { int base, first, n; uint32_t vmask; float total; };
    auto analyse = [&](int w) -> WinInfo {
        WinInfo wi;
        wi.base = window_base(p, w); wi.first = -1; wi.n = 0; wi.vmask = 0u; wi.total = 0.f;
#pragma unroll
        for (int m0 = 0; m0 < WS; m0 += 4) {         // four members' flags and masses in flight (WS >= ws)
            if (m0 >= p.ws) break;
            uint32_t vv[4];
            float mm[4];
            int tk[4];
            bool inb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                inb[u] = m0 + u < p.ws && member_in_grid(p, w, m0 + u);
                tk[u] = inb[u] ? wi.base + p.moff[m0 + u] : wi.base;     // the window's first token is always there
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) vv[u] = vb ? vb[tk[u]] : 1u;
#pragma unroll
            for (int u = 0; u < 4; ++u) mm[u] = mb ? mb[tk[u]] : 1.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (!inb[u] || vv[u] == 0) continue;
                wi.vmask |= 1u << (m0 + u);
                ++wi.n;
                if (wi.first < 0) wi.first = tk[u];
                wi.total += mm[u];
            }
        }
        return wi;
    };
    WinInfo win0 = analyse(min(tid, W - 1));         // nearly always the thread's only window (W <= 1024)
    MD_DTICK(8);

    if (with_keys) {
        // head statistics (m_h, Z_h) and the factor of every group: f[g][h] = exp2(m_g - m_h) / (Z_h * Hc)
        float* s_f = reinterpret_cast<float*>(s_dyn + ((4 * (size_t)M + 15) & ~(size_t)15));   // [gps][PRE], gone before the key flags are written
        {
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < NPB; ++u) {
                if (lane + u * kWave >= gps) pv[u] = make_float2(-INFINITY, 0.f);
                mx = fmaxf(mx, pv[u].x);
            }
            const float gm = wave_max(mx);
            MD_DTICK(9);
            float z = 0.f;
#pragma unroll
            for (int u = 0; u < NPB; ++u) {
                pv[u].x = fast_exp2(pv[u].x - gm);   // (gm is finite: the CLS row always counts)
                z = fmaf(pv[u].y, pv[u].x, z);
            }
            const float inv = wv < p.Hc ? 1.0f / (wave_sum(z) * (float)p.Hc) : 0.f;
#pragma unroll
            for (int u = 0; u < NPB; ++u)
                if (lane + u * kWave < gps) s_f[(lane + u * kWave) * PRE + wv] = pv[u].x * inv;
        }
        if (!EARLY) request_numerators(0);
        MD_DTICK(10);
        __syncthreads();
        MD_DTICK(1);
        // a_cls (head mean of the probabilities) of the tokens tid + 1024*t
        float* s_a = s_tmass;                        // free until the merge decisions
#pragma unroll
        for (int t0 = 0; t0 < IPT; t0 += PT) {
            if (t0 > 0) request_numerators(t0);
#pragma unroll
            for (int t = 0; t < PT; ++t) {
                const int j = tid + 1024 * (t0 + t);
                const f32x4* fr = reinterpret_cast<const f32x4*>(s_f + (size_t)(min(j, M - 1) + 1) / kClsRows * PRE);
                float a = 0.f;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 f = fr[q];
                    a = fmaf(xl[t][q].x, f.x, a);
                    a = fmaf(xl[t][q].y, f.y, a);
                    a = fmaf(xl[t][q].z, f.z, a);
                    a = fmaf(xl[t][q].w, f.w, a);
                }
                if (j < M) s_a[j] = a;
            }
        }
        __syncthreads();
        MD_DTICK(2);
        uint64_t rk[IPT];
        float av[IPT];
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const int j = j0 + t;
            av[t] = s_a[min(j, M - 1)];
            const float a = ok[t] ? av[t] : -INFINITY;
            if (j < M && a_cls_out) a_cls_out[(size_t)b * M + j] = a;
            rk[t] = ok[t] ? rank_key(a, j) : 0ull;
        }
        if (!key_adaptive) {                         // Eq. 7, budget form: the key_budget largest scores
            const SelectBound sb = block_select_topk<IPT>(rk, key_budget, s_hist);
#pragma unroll
            for (int t = 0; t < IPT; ++t) sel[t] = rk[t] != 0 && (rk[t] >> sb.shift) >= sb.bound;
        } else {                                     // Eq. 7 as printed: a_cls > mu, mu = mean + lambda * std
            float s1 = 0.f;
            int cnt = 0;
#pragma unroll
            for (int t = 0; t < IPT; ++t)
                if (ok[t]) { s1 += av[t]; ++cnt; }
            s1 = block_sum(s1, s_redf);
            cnt = block_sum_i(cnt, s_red);
            const float mean = cnt > 0 ? s1 / (float)cnt : 0.f;
            float s2 = 0.f;
#pragma unroll
            for (int t = 0; t < IPT; ++t)
                if (ok[t]) { const float dlt = av[t] - mean; s2 = fmaf(dlt, dlt, s2); }
            s2 = block_sum(s2, s_redf);
            const float mu = mean + key_lambda * sqrtf(cnt > 0 ? s2 / (float)cnt : 0.f);
#pragma unroll
            for (int t = 0; t < IPT; ++t) sel[t] = ok[t] && av[t] > mu;
        }
    } else if (a_cls_out) {
#pragma unroll
        for (int t = 0; t < IPT; ++t)
            if (j0 + t < M) a_cls_out[(size_t)b * M + j0 + t] = 0.f;
    }
    MD_DTICK(3);
#pragma unroll
    for (int t = 0; t < IPT; ++t)
        if (j0 + t < M) { s_key[j0 + t] = sel[t]; s_state[j0 + t] = 0; }
    __syncthreads();
    MD_DTICK(4);

    // ---- merge decision per window: S > tau, >= 2 valid members, no key member.  The window's thread
    // leaves each member's fate (and the merged mass at the first valid member) in LDS, so that the
    // per-token pass below needs no index arithmetic.
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        const int w = tid + 1024 * t;                // windows go round the threads: there are fewer than tokens
        if (w >= W) continue;
        const WinInfo wi = t == 0 ? win0 : analyse(w);
        bool has_key = false;
#pragma unroll
        for (int m = 0; m < WS; ++m)
            if (m < p.ws && ((wi.vmask >> m) & 1u)) has_key |= s_key[wi.base + p.moff[m]] != 0;
        const bool mg = wi.n >= 2 && !has_key && simv[t] > tau;
        if (mg) {
#pragma unroll
            for (int m = 0; m < WS; ++m) {
                if (m >= p.ws || !((wi.vmask >> m) & 1u)) continue;
                const int tok = wi.base + p.moff[m];
                s_state[tok] = tok == wi.first ? 1 : 2;
            }
            s_tmass[wi.first] = wi.total;
        }
        wmerged[(size_t)b * W + w] = mg;
        if (window_sim_out) window_sim_out[(size_t)b * W + w] = simv[t];
    }
    __syncthreads();
    MD_DTICK(5);

    // ---- keys and survivors in ascending token index: one block scan of (keys << 16 | survivors) per thread
    bool surv[IPT], merged[IPT];
    int packed = 0;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        surv[t] = false; merged[t] = false;
        if (ok[t]) {
            const int stt = s_state[j0 + t];
            merged[t] = stt != 0;
            surv[t] = stt != 2;
            if (stt == 1) mass[t] = s_tmass[j0 + t];
        }
        packed += (sel[t] ? 0x10000 : 0) + (surv[t] ? 1 : 0);
    }
    const int incl = wave_incl_scan_i(packed);
    if (lane == kWave - 1) s_red[wv] = incl;
    __syncthreads();
    MD_DTICK(6);
    int total;
    int excl = wave_prefix_of_totals(s_red, total) + incl - packed;
    int kpos = excl >> 16, spos = excl & 0xFFFF;
    const int nkeys = total >> 16, nsurv = total & 0xFFFF;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        const int j = j0 + t;
        if (sel[t]) {
            if (kpos < key_budget) key_index[(size_t)b * key_budget + kpos] = j;
            ++kpos;
        }
        if (j < M) dstpos[(size_t)b * M + j] = surv[t] ? spos : -1;
        if (surv[t]) {
            const size_t o = (size_t)b * M + spos;
            out_index[o] = j;
            out_mass[o] = mass[t];
            out_is_key[o] = merged[t] ? 0 : (sel[t] ? 1 : 0);
            ++spos;
        }
    }
    if (with_keys) {
        for (int r = nkeys + tid; r < key_budget; r += blockDim.x) key_index[(size_t)b * key_budget + r] = -1;
        if (key_count && tid == 0) key_count[b] = nkeys;
    }
    if (tid == 0) out_count[b] = nsurv;
    if (out_valid)
        for (int s2 = tid; s2 < M; s2 += blockDim.x) out_valid[(size_t)b * M + s2] = s2 < nsurv;
#ifdef MD_DECIDE_TICKS
    MD_DTICK(7);
    if (threadIdx.x == 0 && blockIdx.x == 0)
        printf("issue %d gm %d f %d bar %d | acls %d select %d keyflags %d windows %d scan %d writes %d total %d\n",
               (int)(ticks[8] - ticks[0]), (int)(ticks[9] - ticks[8]), (int)(ticks[10] - ticks[9]), (int)(ticks[1] - ticks[10]),
               (int)(ticks[2] - ticks[1]), (int)(ticks[3] - ticks[2]), (int)(ticks[4] - ticks[3]), (int)(ticks[5] - ticks[4]),
               (int)(ticks[6] - ticks[5]), (int)(ticks[7] - ticks[6]), (int)(ticks[7] - ticks[0]));
#endif
}

// ---------------------------------------------------------------------------------------------
// Writes the surviving rows.  One wave per window.
template <bool BF>
__global__ __launch_bounds__(256) void encode_emit_kernel(
    const void* __restrict__ x, const uint8_t* __restrict__ valid, const float* __restrict__ mass_in,
    EncodeDims p, const uint8_t* __restrict__ wmerged, const int32_t* __restrict__ dstpos,
    void* __restrict__ out_x)
{
    constexpr int VEC = Vec<BF>::N;
    const int lane = lane_id();
    const long item = (long)blockIdx.x * (blockDim.x >> 6) + wave_id();
    if (item >= (long)p.B * p.W) return;
    const int b = (int)(item / p.W), w = (int)(item % p.W);
    const size_t esz = BF ? 2 : 4;
    const size_t rowb = (size_t)p.D * esz;
    const char* xb = static_cast<const char*>(x) + (size_t)b * p.M * rowb;
    char* ob = static_cast<char*>(out_x) + (size_t)b * p.M * rowb;
    const uint8_t* vb = valid ? valid + (size_t)b * p.M : nullptr;
    const float* mb = mass_in ? mass_in + (size_t)b * p.M : nullptr;
    const int32_t* dst_b = dstpos + (size_t)b * p.M;

    // lane m < ws: token, validity, destination row and mass of member m, all requested at once
    const int is_merged = wmerged[(size_t)b * p.W + w];
    const int tok_l = lane_member_token(p, w, lane);
    const int ok_l = lane < p.ws && tok_l >= 0 && (!vb || vb[max(tok_l, 0)]);
    const int pos_l = ok_l ? dst_b[tok_l] : -1;
    const float mass_l = ok_l ? (mb ? mb[tok_l] : 1.0f) : 0.f;
    const int nchunk = (int)(rowb / 16);

    if (!is_merged) {
        // plain copies, up to four rows in flight
        for (int m0 = 0; m0 < p.ws; m0 += 4) {
            const u32x4* src[4];
            u32x4* dst[4];
            bool okm[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int m = min(m0 + u, p.ws - 1);
                okm[u] = m0 + u < p.ws && wave_member(ok_l, m) != 0;
                src[u] = reinterpret_cast<const u32x4*>(xb + (size_t)max(wave_member(tok_l, m), 0) * rowb);
                dst[u] = reinterpret_cast<u32x4*>(ob + (size_t)max(wave_member(pos_l, m), 0) * rowb);
            }
            for (int c = lane; c < nchunk; c += kWave) {
                u32x4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src[u] + c);   // unguarded: all in flight
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (okm[u]) __builtin_nontemporal_store(v[u], dst[u] + c);
            }
        }
        return;
    }
    // mass-weighted mean of the valid members (members in ascending order), written at the first one
    const uint64_t okmask = __ballot(ok_l != 0);
    if (okmask == 0ull) return;                      // cannot happen: a merged window has >= 2 valid members
    const int first_m = __builtin_ctzll(okmask);
    float msum = 0.f;
    for (int m = 0; m < p.ws; ++m)
        if ((okmask >> m) & 1ull) msum += __builtin_bit_cast(float, wave_member(__builtin_bit_cast(int, mass_l), m));
    char* orow = ob + (size_t)wave_member(pos_l, first_m) * rowb;
    for (int c = lane * VEC; c < p.D; c += kWave * VEC) {
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
        for (int m0 = 0; m0 < p.ws; m0 += 4) {
            float v[4][VEC], mm[4];
            bool okm[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int m = min(m0 + u, p.ws - 1);
                okm[u] = m0 + u < p.ws && ((okmask >> m) & 1ull);
                mm[u] = __builtin_bit_cast(float, wave_member(__builtin_bit_cast(int, mass_l), m));
                Vec<BF>::load_once(xb + (size_t)max(wave_member(tok_l, m), 0) * rowb, c, v[u]);   // unguarded, see above
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (!okm[u]) continue;
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fmaf(mm[u], v[u][e], acc[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = acc[e] / msum;
        Vec<BF>::store(orow, c, acc);
    }
}

struct EncodeWorkspace {
    float* logits; float2* cls_part; float* acls; float* sim; uint8_t* iskey; uint8_t* wmerged; int32_t* dstpos;
    size_t bytes;
};

EncodeWorkspace carve_encode(void* base, int B, int M, int W, int Hc) {
    Carver c(base);
    EncodeWorkspace ws;
    ws.logits = c.take<float>((size_t)B * (Hc > 0 ? Hc : 1) * (M + 1));
    ws.cls_part = c.take<float2>((size_t)B * (Hc > 0 ? Hc : 1) * cls_groups(M));
    ws.acls = c.take<float>((size_t)B * M);
    ws.sim = c.take<float>((size_t)B * W);
    ws.iskey = c.take<uint8_t>((size_t)B * M);
    ws.wmerged = c.take<uint8_t>((size_t)B * W);
    ws.dstpos = c.take<int32_t>((size_t)B * M);
    ws.bytes = c.off;
    return ws;
}

// Dynamic LDS of the fast decision kernel: [M] floats, then the larger of ([M] + [M] flag bytes) and the
// [groups][16] factors (16-byte aligned).
size_t decide_fast_lds_bytes(int M) {
    const size_t head = (4 * (size_t)M + 15) & ~(size_t)15;
    const size_t factors = (size_t)cls_groups(M) * 16 * 4, flags = 2 * (size_t)M + 16;
    return head + (factors > flags ? factors : flags);
}
// More than 64 KiB of dynamic LDS has to be asked for (only the 8-tokens-per-thread form needs it).
bool decide_fast_lds_ready(int M, size_t bytes) {
    if (bytes <= 64 * 1024) return true;
    if (M <= 4096) return false;
    bool ok = true;
    ok &= hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_decide_fast_kernel<8, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
    ok &= hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_decide_fast_kernel<8, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
    ok &= hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_decide_fast_kernel<8, 16>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
    return ok;
}

template <int WSM>
void launch_scores(dim3 grid, hipStream_t st, bool xbf, bool qkbf, const void* x, const void* q_cls, const void* k_cls,
                   const uint8_t* valid, const EncodeDims& p, int with_cls, float* sim, float* logits, float2* cls_part) {
    if (xbf && qkbf) MD_LAUNCH("encode_scores", st, (encode_scores_kernel<WSM, true, true>), grid, 64 * kEncWaves, 0, x, q_cls, k_cls, valid, p, with_cls, sim, logits, cls_part);
    else if (xbf) MD_LAUNCH("encode_scores", st, (encode_scores_kernel<WSM, true, false>), grid, 64 * kEncWaves, 0, x, q_cls, k_cls, valid, p, with_cls, sim, logits, cls_part);
    else if (qkbf) MD_LAUNCH("encode_scores", st, (encode_scores_kernel<WSM, false, true>), grid, 64 * kEncWaves, 0, x, q_cls, k_cls, valid, p, with_cls, sim, logits, cls_part);
    else MD_LAUNCH("encode_scores", st, (encode_scores_kernel<WSM, false, false>), grid, 64 * kEncWaves, 0, x, q_cls, k_cls, valid, p, with_cls, sim, logits, cls_part);
}

}  // namespace
}  // namespace md

using namespace md;

extern "C" size_t mustdrop_encode_merge_workspace_bytes(int B, int T, int Hg, int Wg, int Hc, int kt, int kh, int kw) {
    if (B <= 0 || T <= 0 || Hg <= 0 || Wg <= 0 || kt <= 0 || kh <= 0 || kw <= 0) return 0;
    const long M = (long)T * Hg * Wg;
    const long W = (long)((T + kt - 1) / kt) * ((Hg + kh - 1) / kh) * ((Wg + kw - 1) / kw);
    return carve_encode(nullptr, B, (int)M, (int)W, Hc).bytes;
}

namespace md {
namespace {
// Both forms of the key set (Eq. 7): key_adaptive == 0: the key_budget largest scores; key_adaptive == 1:
// a_cls > mean + key_lambda * std, key_budget = capacity of key_index, key_count = size of the set.
int encode_merge_impl(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_adaptive, int key_budget, float key_lambda,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index, int32_t* key_count,
    float* a_cls_out, float* window_sim_out,
    void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    if (x_dtype != MD_F32 && x_dtype != MD_BF16) return fail(MD_EDTYPE, "encode_merge: unknown x_dtype %d", (int)x_dtype);
    if (B <= 0 || T <= 0 || Hg <= 0 || Wg <= 0 || D <= 0)
        return fail(MD_EINVAL, "encode_merge: B, T, Hg, Wg, D must be positive (got %d %d %d %d %d)", B, T, Hg, Wg, D);
    if (kt <= 0 || kh <= 0 || kw <= 0) return fail(MD_EINVAL, "encode_merge: window sizes must be positive");
    const long ws_l = (long)kt * kh * kw;
    if (ws_l > kMaxWindow) return fail(MD_ESHAPE, "encode_merge: window of %ld tokens exceeds the limit of %d", ws_l, kMaxWindow);
    const long M_l = (long)T * Hg * Wg;
    if (M_l > (1l << 24) || (long)B * M_l > (1l << 30)) return fail(MD_ESHAPE, "encode_merge: too many tokens");
    const int nwt = (T + kt - 1) / kt, nwy = (Hg + kh - 1) / kh, nwx = (Wg + kw - 1) / kw;   // border windows are clipped
    const int M = (int)M_l, ws = (int)ws_l, W = nwt * nwy * nwx;
    if (key_budget < 0 || (!key_adaptive && key_budget > M))
        return fail(MD_EINVAL, "encode_merge: key_budget %d outside [0, %d]", key_budget, M);
    if (key_adaptive && (std::isnan(key_lambda) || !key_count))
        return fail(MD_EINVAL, "encode_merge: the adaptive key rule needs a key_lambda that is a number and key_count");
    const bool with_keys = key_adaptive || key_budget > 0;
    if (!x || !out_x || !out_index || !out_mass || !out_is_key || !out_count)
        return fail(MD_EINVAL, "encode_merge: x and the out_* arrays are required");
    if (std::isnan(tau)) return fail(MD_EINVAL, "encode_merge: tau is NaN");
    const size_t xe = elt_size(x_dtype);
    if ((D * xe) % 16) return fail(MD_EALIGN, "encode_merge: a row of D=%d elements is not a multiple of 16 bytes", D);
    if (!aligned16(x) || !aligned16(out_x)) return fail(MD_EALIGN, "encode_merge: x / out_x must be 16-byte aligned");
    if (with_keys) {
        if (qk_dtype != MD_F32 && qk_dtype != MD_BF16) return fail(MD_EDTYPE, "encode_merge: unknown qk_dtype %d", (int)qk_dtype);
        if (!q_cls || !k_cls || (key_budget > 0 && !key_index))
            return fail(MD_EINVAL, "encode_merge: q_cls, k_cls (and key_index, if it has room) are required when keys are selected");
        if (Hc <= 0 || dc <= 0) return fail(MD_EINVAL, "encode_merge: Hc and dc must be positive");
        if (Hc > kMaxClsHeads) return fail(MD_ESHAPE, "encode_merge: Hc=%d exceeds the limit of %d", Hc, kMaxClsHeads);
        if ((long)Hc * dc != D) return fail(MD_ESHAPE, "encode_merge: Hc*dc = %ld differs from D = %d", (long)Hc * dc, D);
        const int vec = qk_dtype == MD_BF16 ? 8 : 4;
        if ((dc & (dc - 1)) || dc < vec) return fail(MD_ESHAPE, "encode_merge: dc=%d must be a power of two >= %d", dc, vec);
        if (!aligned16(q_cls) || !aligned16(k_cls)) return fail(MD_EALIGN, "encode_merge: q_cls / k_cls must be 16-byte aligned");
    } else if (q_cls || k_cls) {
        return fail(MD_EINVAL, "encode_merge: q_cls / k_cls given but key_budget == 0");
    }
    const size_t xbytes = (size_t)B * M * D * xe;
    if (overlaps(x, xbytes, out_x, xbytes)) return fail(MD_EALIAS, "encode_merge: out_x overlaps x");
    const EncodeWorkspace wsp = carve_encode(workspace, B, M, W, with_keys ? Hc : 0);
    if (!workspace || workspace_bytes < wsp.bytes)
        return fail(MD_EWORKSPACE, "encode_merge: workspace of %zu bytes needed, %zu given", wsp.bytes, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(MD_EALIGN, "encode_merge: workspace must be 256-byte aligned");

    EncodeDims p;
    p.B = B; p.T = T; p.Hg = Hg; p.Wg = Wg; p.D = D; p.Hc = with_keys ? Hc : 0; p.dc = dc;
    p.kt = kt; p.kh = kh; p.kw = kw; p.M = M; p.W = W; p.ws = ws;
    p.nwx = nwx; p.nwy = nwy; p.nwt = nwt;
    p.clipped = (T % kt || Hg % kh || Wg % kw) ? 1 : 0;
    for (int m = 0; m < kMaxWindow; ++m) p.moff[m] = m < ws ? member_offset(p, m) : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);

    const long items = (long)B * W + (with_keys ? (long)B * cls_groups(M) : 0);
    dim3 sgrid((unsigned)((items + kEncWaves - 1) / kEncWaves));
    const bool xbf = x_dtype == MD_BF16, qkbf = qk_dtype == MD_BF16;
    const int with_cls = with_keys;
    if (ws <= 2) launch_scores<2>(sgrid, st, xbf, qkbf, x, q_cls, k_cls, valid, p, with_cls, wsp.sim, wsp.logits, wsp.cls_part);
    else if (ws <= 4) launch_scores<4>(sgrid, st, xbf, qkbf, x, q_cls, k_cls, valid, p, with_cls, wsp.sim, wsp.logits, wsp.cls_part);
    else if (ws <= 8) launch_scores<8>(sgrid, st, xbf, qkbf, x, q_cls, k_cls, valid, p, with_cls, wsp.sim, wsp.logits, wsp.cls_part);
    else launch_scores<16>(sgrid, st, xbf, qkbf, x, q_cls, k_cls, valid, p, with_cls, wsp.sim, wsp.logits, wsp.cls_part);
    dim3 wgrid((unsigned)(((long)B * W + kEncWaves - 1) / kEncWaves));
    const size_t dlds = decide_fast_lds_bytes(M);
    const bool fast_ok = M <= 8192 && (!with_keys || (Hc <= 16 && Hc % 4 == 0)) && decide_fast_lds_ready(M, dlds);
#define MD_DECIDE_FAST(IPT_, WS_)                                                                             \
    MD_LAUNCH("encode_decide", st, (encode_decide_fast_kernel<IPT_, WS_>), B, 1024, dlds,                  \
        p, valid, mass_in, wsp.logits, wsp.cls_part, wsp.sim, tau, key_budget, key_adaptive, key_lambda, key_count,  \
        wsp.wmerged, wsp.dstpos,                                                                                   \
        out_index, out_mass, out_is_key, out_valid, out_count, key_index, a_cls_out, window_sim_out)
#define MD_DECIDE_FAST_WS(IPT_)                                                                               \
    do { if (ws <= 4) MD_DECIDE_FAST(IPT_, 4); else if (ws <= 8) MD_DECIDE_FAST(IPT_, 8); else MD_DECIDE_FAST(IPT_, 16); } while (0)
    if (fast_ok && M <= 1024) MD_DECIDE_FAST_WS(1);
    else if (fast_ok && M <= 2048) MD_DECIDE_FAST_WS(2);
    else if (fast_ok && M <= 3072) MD_DECIDE_FAST_WS(3);     // e.g. five tiles of 24 x 24 tokens
    else if (fast_ok && M <= 4096) MD_DECIDE_FAST_WS(4);
    else if (fast_ok && M <= 5120) MD_DECIDE_FAST_WS(5);     // e.g. eight frames of 24 x 24 tokens
    else if (fast_ok && M <= 6144) MD_DECIDE_FAST_WS(6);
    else if (fast_ok) MD_DECIDE_FAST_WS(8);
    else
        MD_LAUNCH("encode_decide", st, (encode_decide_kernel), B, 1024, 0,
            p, valid, mass_in, wsp.logits, wsp.cls_part, wsp.sim, tau, key_budget, key_adaptive, key_lambda, key_count,
            wsp.acls, wsp.iskey, wsp.wmerged, wsp.dstpos,
            out_index, out_mass, out_is_key, out_valid, out_count, key_index, a_cls_out, window_sim_out);
#undef MD_DECIDE_FAST_WS
#undef MD_DECIDE_FAST
    if (x_dtype == MD_BF16) MD_LAUNCH("encode_emit", st, (encode_emit_kernel<true>), wgrid, 64 * kEncWaves, 0, x, valid, mass_in, p, wsp.wmerged, wsp.dstpos, out_x);
    else MD_LAUNCH("encode_emit", st, (encode_emit_kernel<false>), wgrid, 64 * kEncWaves, 0, x, valid, mass_in, p, wsp.wmerged, wsp.dstpos, out_x);
    return check_launch("encode_merge");
}
}  // namespace
}  // namespace md

extern "C" int mustdrop_encode_merge(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_budget,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index,
    float* a_cls_out, float* window_sim_out,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return encode_merge_impl(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, tau,
                             0, key_budget, 0.f, out_x, out_index, out_mass, out_is_key, out_valid, out_count,
                             key_index, nullptr, a_cls_out, window_sim_out, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// The same stage for callers that cannot hand over (or allocate) a workspace: the scratch memory is a
// file-scope device array.  Every GPU the library runs on holds its own copy at its own address; the
// host-side name of the array is only a handle, the address a kernel can use comes from
// hipGetSymbolAddress (once per device, kept).
static __device__ __align__(256) unsigned char scratch[MUSTDROP_STATIC_SCRATCH_BYTES];

namespace md {
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (resolved at the first call on that device).
int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(MD_EHIP, "encode_merge_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(MD_EHIP, "encode_merge_noalloc: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(MD_EHIP, "encode_merge_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MD_OK;
}
}  // namespace
}  // namespace md

extern "C" int mustdrop_encode_merge_noalloc(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_budget,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index,
    float* a_cls_out, float* window_sim_out, void* stream)
{
    clear_error();
    if (B <= 0 || T <= 0 || Hg <= 0 || Wg <= 0 || kt <= 0 || kh <= 0 || kw <= 0)
        return fail(MD_EINVAL, "encode_merge_noalloc: B, T, Hg, Wg and the window sizes must be positive");
    if ((long)T * Hg * Wg > (1l << 24) || (long)B * T * Hg * Wg > (1l << 30))
        return fail(MD_ESHAPE, "encode_merge_noalloc: too many tokens");
    const size_t need = mustdrop_encode_merge_workspace_bytes(B, T, Hg, Wg, key_budget > 0 ? Hc : 0, kt, kh, kw);
    if (need > (size_t)MUSTDROP_STATIC_SCRATCH_BYTES)
        return fail(MD_EWORKSPACE, "encode_merge_noalloc: this shape needs %zu bytes of scratch memory, the static buffer holds %zu; "
                    "use mustdrop_encode_merge with a workspace", need, (size_t)MUSTDROP_STATIC_SCRATCH_BYTES);
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != MD_OK) return rc;
    return encode_merge_impl(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, tau,
                             0, key_budget, 0.f, out_x, out_index, out_mass, out_is_key, out_valid, out_count,
                             key_index, nullptr, a_cls_out, window_sim_out, ptr, (size_t)MUSTDROP_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int mustdrop_encode_merge_adaptive(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, float key_lambda, int key_cap,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index, int32_t* key_count,
    float* a_cls_out, float* window_sim_out,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return encode_merge_impl(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, tau,
                             1, key_cap, key_lambda, out_x, out_index, out_mass, out_is_key, out_valid, out_count,
                             key_index, key_count, a_cls_out, window_sim_out, workspace, workspace_bytes, stream);
}
