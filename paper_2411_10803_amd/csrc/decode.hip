// Stage 3 -- decode (Sec. 3.5): score the KV cache against the query of the token being generated
// (attention of Eq. 4), keep a running score per entry, evict down to a budget and compact the
// cache by hole filling.
//
//   decode_logits_kernel  one wave per cache entry at a time: an entry's K row (H heads x d, all
//                         contiguous) is read once with 16-byte loads, 16 lanes per head slice;
//                         segmented butterflies give the H logits.  Pure streaming: a GEMV at about
//                         1 flop per byte, so plain ALUs, not MFMA.
//   decode_select_kernel  one block per sample: softmax statistics per head, head mean, running
//                         score update, radix top-k among unprotected entries, hole/mover lists,
//                         moves of the small per-entry arrays
//   decode_move_kernel    copies the K and V rows of the movers into the holes
#include "md_device.hpp"
#include "md_host.hpp"

namespace md {
namespace {

constexpr float kLog2eD = 1.4426950408889634f;

struct DecodeDims { int B, Lcap, H, d; };
constexpr int kMaxStatParts = 256;               // blocks per sample of the streaming logits kernel

// logits[b][j][h] = scale * q[b][h] . k[b][j][h]      (token-major so an entry's H logits are contiguous)
// LPH = lanes per head slice = d / 8.  Generic shape: walks an entry's row in 1 KiB pieces.
template <int LPH>
__global__ __launch_bounds__(256) void decode_logits_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_cache, const int32_t* __restrict__ len,
    DecodeDims p, KvLayout lay, float scale, int tokens_per_block, float* __restrict__ logits)
{
    const int lane = lane_id(), wv = wave_id();
    const int b = blockIdx.y;
    const int n = min(len[b], p.Lcap);
    const int t0 = blockIdx.x * tokens_per_block;
    if (t0 >= n) return;
    const int t1 = min(t0 + tokens_per_block, n);
    const int row = p.H * p.d;                      // elements per entry
    const int nvec = row / 8;                       // 16-byte vectors per entry
    const int iters = (nvec + kWave - 1) / kWave;
    const uint16_t* qb = q + (long)b * row;
    const uint16_t* kb = k_cache + (long)b * lay.batch;
    float* lb = logits + (long)b * p.Lcap * p.H;

    for (int it = 0; it < iters; ++it) {
        const int idx = it * kWave + lane;
        float qv[8];
        if (idx < nvec) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(qb + idx * 8);
            qv[0] = bf16_lo(w.x); qv[1] = bf16_hi(w.x); qv[2] = bf16_lo(w.y); qv[3] = bf16_hi(w.y);
            qv[4] = bf16_lo(w.z); qv[5] = bf16_hi(w.z); qv[6] = bf16_lo(w.w); qv[7] = bf16_hi(w.w);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[e] = 0.f;
        }
        const int head = idx / LPH;
        const long in_row = (long)head * lay.head + (idx % LPH) * 8;      // dense: idx * 8
        for (int j = t0 + wv; j < t1; j += 4) {
            float part = 0.f;
            if (idx < nvec) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(kb + (long)j * lay.token + in_row);
                part = qv[0] * bf16_lo(w.x);
                part = fmaf(qv[1], bf16_hi(w.x), part);
                part = fmaf(qv[2], bf16_lo(w.y), part);
                part = fmaf(qv[3], bf16_hi(w.y), part);
                part = fmaf(qv[4], bf16_lo(w.z), part);
                part = fmaf(qv[5], bf16_hi(w.z), part);
                part = fmaf(qv[6], bf16_lo(w.w), part);
                part = fmaf(qv[7], bf16_hi(w.w), part);
            }
            part = group_sum<LPH>(part);
            if (idx < nvec && (lane & (LPH - 1)) == 0) lb[(long)j * p.H + head] = part * scale;
        }
    }
}

__device__ __forceinline__ float dot8(const u32x4& a, const float (&qv)[8]) {
    float s = qv[0] * bf16_lo(a.x);
    s = fmaf(qv[1], bf16_hi(a.x), s);
    s = fmaf(qv[2], bf16_lo(a.y), s);
    s = fmaf(qv[3], bf16_hi(a.y), s);
    s = fmaf(qv[4], bf16_lo(a.z), s);
    s = fmaf(qv[5], bf16_hi(a.z), s);
    s = fmaf(qv[6], bf16_lo(a.w), s);
    s = fmaf(qv[7], bf16_hi(a.w), s);
    return s;
}

// Streaming shape: an entry's row is NIT KiB (H*d*2 = NIT*1024 bytes).  A wave keeps the whole query
// in registers and reads each entry's row in one go: NIT independent 16-byte loads per lane, every
// load instruction covering 1 KiB of consecutive addresses.  Waves stride over the sample's entries.
// Each wave also keeps online softmax statistics (max, sum of exp2) of every head over the entries
// it has seen; the block's four waves are merged and written as one partial per (sample, block, head),
// so the selection kernel does not have to sweep the logits for them.
// STRIDED: the cache has another layout; a load instruction then covers kWave/LPH head slices of
// d*2 contiguous bytes each instead of 1 KiB of one row.
// STREAM_ONCE: the cache is larger than what the L2 / Infinity Cache can hold until the row moves, so
// the K rows are read with streaming loads (they would only evict each other and everything else).
template <int LPH, int NIT, bool STRIDED, bool STREAM_ONCE>
__global__ __launch_bounds__(256) void decode_logits_stream_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_cache, const int32_t* __restrict__ len,
    DecodeDims p, KvLayout lay, float scale, float* __restrict__ logits, float2* __restrict__ stat_partial)
{
    constexpr int HPI = kWave / LPH;                 // heads per load instruction
    __shared__ float s_m[4][NIT * HPI], s_z[4][NIT * HPI];
    const int lane = lane_id(), wv = wave_id();
    const int b = blockIdx.y;
    const int wave_global = blockIdx.x * 4 + wv;
    const int nwaves = gridDim.x * 4;
    const int row = p.H * p.d;
    const u32x4* qb = reinterpret_cast<const u32x4*>(q + (long)b * row);
    const u32x4* kb = reinterpret_cast<const u32x4*>(k_cache + (long)b * p.Lcap * row);
    const uint16_t* ks = k_cache + (long)b * lay.batch;
    long off[NIT];                                   // STRIDED: element offset of this lane's vectors within an entry
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int idx = it * kWave + lane;
        off[it] = (long)(idx / LPH) * lay.head + (idx % LPH) * 8;
    }
    float* lb = logits + (long)b * p.Lcap * p.H;
    const float scale_l2 = scale * kLog2eD;

    float qv[NIT][8];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const u32x4 w = qb[it * kWave + lane];
        qv[it][0] = bf16_lo(w.x); qv[it][1] = bf16_hi(w.x); qv[it][2] = bf16_lo(w.y); qv[it][3] = bf16_hi(w.y);
        qv[it][4] = bf16_lo(w.z); qv[it][5] = bf16_hi(w.z); qv[it][6] = bf16_lo(w.w); qv[it][7] = bf16_hi(w.w);
    }
    float m[NIT], z[NIT];                            // log2 domain; every lane of a head's group holds the same values
#pragma unroll
    for (int it = 0; it < NIT; ++it) { m[it] = -INFINITY; z[it] = 0.f; }

    const int n = min(max(len[b], 0), p.Lcap);
    for (int j = wave_global; j < n; j += nwaves) {
        u32x4 kv[NIT];
        if constexpr (STRIDED) {
            const uint16_t* kr = ks + (long)j * lay.token;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const u32x4* src = reinterpret_cast<const u32x4*>(kr + off[it]);
                kv[it] = STREAM_ONCE ? __builtin_nontemporal_load(src) : *src;
            }
        } else {
            const u32x4* kr = kb + (long)j * (row / 8);
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                kv[it] = STREAM_ONCE ? __builtin_nontemporal_load(kr + it * kWave + lane) : kr[it * kWave + lane];
        }
        float part[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) part[it] = dot8(kv[it], qv[it]);
#pragma unroll
        for (int it = 0; it < NIT; ++it) part[it] = group_sum<LPH>(part[it]);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const float t2 = part[it] * scale_l2;
            const float dlt = t2 - m[it];            // +inf on the first entry
            const float e = fast_exp2(-fabsf(dlt));
            z[it] = dlt > 0.f ? fmaf(z[it], e, 1.0f) : z[it] + e;
            m[it] = fmaxf(m[it], t2);
        }
        if ((lane & (LPH - 1)) == 0) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) lb[(long)j * p.H + it * HPI + lane / LPH] = part[it] * scale;
        }
    }
    if ((lane & (LPH - 1)) == 0) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) { s_m[wv][it * HPI + lane / LPH] = m[it]; s_z[wv][it * HPI + lane / LPH] = z[it]; }
    }
    __syncthreads();
    for (int h = threadIdx.x; h < NIT * HPI; h += blockDim.x) {
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, s_m[w][h]);
        float zn = 0.f;
        if (mn > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) zn += s_z[w][h] * fast_exp2(s_m[w][h] - mn);
        }
        stat_partial[((long)b * gridDim.x + blockIdx.x) * p.H + h] = make_float2(mn, zn);
    }
}

// Selection with everything in registers.  Entries are dealt round-robin: thread t owns the entries
// t, t+1024, ... (coalesced loads; the first one does not depend on the live length, so it is
// requested before the length arrives).  IPT >= ceil(Lcap / 1024).  One round of global loads for
// the common case, then block-level phases only.
template <int IPT, int LPE>
__global__ __launch_bounds__(1024) void decode_select_fast_kernel(
    DecodeDims p, const float* __restrict__ logits, const float2* __restrict__ stat_partial, int n_part,
    float decay, int budget,
    float* __restrict__ acc, int32_t* __restrict__ ids, uint8_t* __restrict__ protect, int32_t* __restrict__ len,
    int32_t* __restrict__ holes, int32_t* __restrict__ movers, int32_t* __restrict__ n_move,
    int32_t* __restrict__ evicted_ids, int32_t* __restrict__ evicted_count)
{
    extern __shared__ int s_holes[];                 // [Lcap] evicted slots below the new length, then [Lcap] a_t
    float* s_at = reinterpret_cast<float*>(s_holes + p.Lcap);
    __shared__ float s_cm[1024], s_cz[1024];         // per head: max (log2 domain), 1 / (Z * H)
    __shared__ int s_red[16];
    __shared__ int s_hist[kSelectHistInts];
    __shared__ uint64_t s_red64[16];
    const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    if (tid < 256) s_hist[tid] = 0;                  // for block_select_topk, after later barriers
    const int H = p.H;
    const float* lb = logits + (long)b * p.Lcap * H;
    float* ab = acc + (long)b * p.Lcap;
    int32_t* ib = ids + (long)b * p.Lcap;
    uint8_t* pb = protect + (long)b * p.Lcap;
    int32_t* hb = holes + (long)b * p.Lcap;
    int32_t* mvb = movers + (long)b * p.Lcap;

    // ---- requests that do not depend on the live length
    float a_old[IPT];
    int id[IPT];
    bool prot[IPT], live[IPT];
    // Logits are read the way they lie in memory: a wave takes 64 consecutive entries (64*H floats)
    // with LPE = H/4 fully coalesced 16-byte loads per lane; lane l then holds heads 4*(l%LPE)..+3 of
    // the entries u*(64/LPE) + l/LPE, u = 0..LPE-1.
    constexpr int PFR = IPT < 2 ? IPT : 2;           // rounds requested before the length is known
    constexpr int EPI = kWave / LPE;                 // entries per load instruction
    f32x4 lpf[PFR][LPE];
#pragma unroll
    for (int t = 0; t < PFR; ++t) {
        const int j = tid + t * 1024;
        const bool in = j < p.Lcap;                  // readable whatever the live length is
        a_old[t] = in ? ab[j] : 0.f;
        id[t] = in ? ib[j] : 0;
        prot[t] = in ? pb[j] != 0 : false;
        const int base = t * 1024 + wv * kWave;
#pragma unroll
        for (int u = 0; u < LPE; ++u) {
            const int e = base + u * EPI + lane / LPE;
            lpf[t][u] = e < p.Lcap ? reinterpret_cast<const f32x4*>(lb + (long)base * H)[u * kWave + lane]
                                   : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // the logits kernel's partial statistics: `parts` consecutive lanes share a head, each takes a slice
    const int parts = min(1024 / H, kWave), sh = tid / parts, sq = tid % parts;
    float mn = -INFINITY, zn = 0.f;
    if (sh < H) {
        const float2* sp = stat_partial + (long)b * n_part * H + sh;
        for (int c = sq; c < n_part; c += parts) {
            const float2 v = sp[(long)c * H];
            const float m2 = fmaxf(mn, v.x);
            if (m2 > -INFINITY) zn = zn * fast_exp2(mn - m2) + v.y * fast_exp2(v.x - m2);
            mn = m2;
        }
    }
    const int n = min(max(len[b], 0), p.Lcap);
    if (n == 0) {
        if (tid == 0) { n_move[b] = 0; if (evicted_count) evicted_count[b] = 0; }
        return;
    }
#pragma unroll
    for (int t = 0; t < PFR; ++t) {
        live[t] = tid + t * 1024 < n;
        if (!live[t]) { prot[t] = false; a_old[t] = 0.f; }
    }
#pragma unroll
    for (int t = PFR; t < IPT; ++t) {                // further rounds only for long caches
        const int j = tid + t * 1024;
        live[t] = j < n;
        a_old[t] = live[t] ? ab[j] : 0.f;
        id[t] = live[t] ? ib[j] : 0;
        prot[t] = live[t] ? pb[j] != 0 : false;
    }
    // the lanes of a head finish the merge: group maximum, then the group sum of the rescaled sums
    {
        float gm = mn;
        if (parts >= 2) gm = fmaxf(gm, dpp_f<0xB1>(gm));
        if (parts >= 4) gm = fmaxf(gm, dpp_f<0x4E>(gm));
        if (parts >= 8) gm = fmaxf(gm, dpp_f<0x141>(gm));
        if (parts >= 16) gm = fmaxf(gm, dpp_f<0x140>(gm));
        if (parts >= 32) gm = fmaxf(gm, __shfl_xor(gm, 16, kWave));
        if (parts >= 64) gm = fmaxf(gm, __shfl_xor(gm, 32, kWave));
        const float zs = group_sum_rt(gm > -INFINITY ? zn * fast_exp2(mn - gm) : 0.f, parts);
        if (sh < H && sq == 0) { s_cm[sh] = gm; s_cz[sh] = __frcp_rn(zs * (float)H); }
    }
    __syncthreads();
    // a_t[j] = mean_h softmax; acc <- decay*acc + a_t.  A lane always works on the same four heads,
    // so their statistics sit in registers; LPE lanes add up an entry's heads and one of them drops
    // the result in LDS, from where the entry's owner picks it up (same wave: LDS keeps program order).
    float a_new[IPT];
    {
        float cm[4], cz[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) { cm[c] = s_cm[4 * (lane % LPE) + c]; cz[c] = s_cz[4 * (lane % LPE) + c]; }
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            a_new[t] = 0.f;
            if (t * 1024 >= n) continue;             // block-uniform: no entries in this round
            const int base = t * 1024 + wv * kWave;
#pragma unroll
            for (int u = 0; u < LPE; ++u) {
                const int e = base + u * EPI + lane / LPE;
                f32x4 v;
                if (t < PFR) v = lpf[t < PFR ? t : 0][u];
                else v = e < n ? reinterpret_cast<const f32x4*>(lb + (long)base * H)[u * kWave + lane] : f32x4{0.f, 0.f, 0.f, 0.f};
                float part = fast_exp2(fmaf(v.x, kLog2eD, -cm[0])) * cz[0];
                part = fmaf(fast_exp2(fmaf(v.y, kLog2eD, -cm[1])), cz[1], part);
                part = fmaf(fast_exp2(fmaf(v.z, kLog2eD, -cm[2])), cz[2], part);
                part = fmaf(fast_exp2(fmaf(v.w, kLog2eD, -cm[3])), cz[3], part);
                part = group_sum<LPE>(part);
                if (lane % LPE == 0 && e < p.Lcap) s_at[e] = part;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int j = tid + t * 1024;
            a_new[t] = live[t] ? fmaf(decay, a_old[t], s_at[j]) : 0.f;
        }
    }
    int np = 0;
#pragma unroll
    for (int t = 0; t < IPT; ++t) np += prot[t];
    np = block_sum_i(np, s_red);

    if (n <= budget) {                               // nothing leaves: only the scores change
#pragma unroll
        for (int t = 0; t < IPT; ++t) if (live[t]) ab[tid + t * 1024] = a_new[t];
        if (tid == 0) { n_move[b] = 0; if (evicted_count) evicted_count[b] = 0; }
        return;
    }
    const int nu = n - np;
    const int extra = min(max(budget - np, 0), nu);
    const int new_len = np + extra;
    uint64_t key[IPT];
#pragma unroll
    for (int t = 0; t < IPT; ++t) key[t] = (live[t] && !prot[t]) ? rank_key(a_new[t], id[t]) : 0ull;

    if (nu - extra == 1) {
        // Steady state of a decode loop: exactly one entry leaves -- the smallest key.  If it is not
        // the last live slot, the last entry (a survivor) moves into its place.
        uint64_t mine = ~0ull;
        int mine_slot = 0;
#pragma unroll
        for (int t = 0; t < IPT; ++t) if (key[t] != 0 && key[t] < mine) { mine = key[t]; mine_slot = tid + t * 1024; }
        const uint64_t victim = block_min_u64(mine, s_red64);
        __shared__ int s_vslot;
        if (mine == victim) s_vslot = mine_slot;     // keys are unique: one writer
        __syncthreads();
        const int vslot = s_vslot, last = n - 1;
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const int j = tid + t * 1024;
            if (!live[t]) continue;
            if (j == vslot) {
                if (evicted_ids) evicted_ids[(long)b * p.Lcap] = id[t];
                if (j == last) ab[j] = a_new[t];     // stays behind the new end, as the oracle leaves it
            } else if (j == last && vslot != last) {
                ab[vslot] = a_new[t]; ib[vslot] = id[t]; pb[vslot] = prot[t] ? 1 : 0;
                ab[j] = a_new[t];
                hb[0] = vslot; mvb[0] = last;
            } else {
                ab[j] = a_new[t];
            }
        }
        if (tid == 0) {
            n_move[b] = vslot != last ? 1 : 0;
            len[b] = new_len;
            if (evicted_count) evicted_count[b] = 1;
        }
        return;
    }

    const SelectBound sb = block_select_topk<IPT>(key, extra, s_hist);
    bool keep[IPT];
#pragma unroll
    for (int t = 0; t < IPT; ++t)
        keep[t] = live[t] && (prot[t] || (extra > 0 && (key[t] >> sb.shift) >= sb.bound));
    // hole / mover / evicted lists in ascending slot order: one pass of block scans per round of entries
    int run_h = 0, run_m = 0, run_e = 0;
    int mrank[IPT];
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        mrank[t] = -1;
        if (t * 1024 >= n) continue;                 // block-uniform
        const int j = tid + t * 1024;
        const bool is_hole = live[t] && !keep[t] && j < new_len;
        const bool is_mover = live[t] && keep[t] && j >= new_len;
        const bool is_ev = live[t] && !keep[t];
        int tot_hm, tot_e;
        const int pre_hm = block_exscan_i((is_hole ? 1 : 0) | (is_mover ? 1 << 16 : 0), s_red, tot_hm);
        const int pre_e = block_exscan_i(is_ev ? 1 : 0, s_red, tot_e);
        if (is_hole) { const int r = run_h + (pre_hm & 0xFFFF); s_holes[r] = j; hb[r] = j; }
        if (is_mover) { mrank[t] = run_m + (pre_hm >> 16); mvb[mrank[t]] = j; }
        if (is_ev && evicted_ids) evicted_ids[(long)b * p.Lcap + run_e + pre_e] = id[t];
        run_h += tot_hm & 0xFFFF; run_m += tot_hm >> 16; run_e += tot_e;
    }
    __syncthreads();
    // write the scores back; a mover's state goes straight to its hole (no overlap: holes < new_len <= movers)
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        const int j = tid + t * 1024;
        if (!live[t]) continue;
        if (mrank[t] >= 0) {
            const int dst = s_holes[mrank[t]];
            ab[dst] = a_new[t];
            ib[dst] = id[t];
            pb[dst] = prot[t] ? 1 : 0;
            ab[j] = a_new[t];
        } else if (keep[t] || j >= new_len) {
            ab[j] = a_new[t];
        }
    }
    if (tid == 0) {
        n_move[b] = run_m;
        len[b] = new_len;
        if (evicted_count) evicted_count[b] = run_e;
    }
}

__global__ __launch_bounds__(1024) void decode_select_kernel(
    DecodeDims p, const float* __restrict__ logits, float decay, int budget,
    float* __restrict__ acc, int32_t* __restrict__ ids, uint8_t* __restrict__ protect, int32_t* __restrict__ len,
    uint8_t* __restrict__ keep, int32_t* __restrict__ holes, int32_t* __restrict__ movers, int32_t* __restrict__ n_move,
    int32_t* __restrict__ evicted_ids, int32_t* __restrict__ evicted_count)
{
    extern __shared__ float s_dyn[];                 // [2*H] max / inv, then [32][H] scratch
    __shared__ int s_red[16];
    __shared__ int s_hist[256];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int H = p.H;
    const int n = min(max(len[b], 0), p.Lcap);
    float* s_max = s_dyn;
    float* s_inv = s_dyn + H;
    float* s_part = s_dyn + 2 * H;                   // [parts][H]
    const float* lb = logits + (long)b * p.Lcap * H;
    float* ab = acc + (long)b * p.Lcap;
    int32_t* ib = ids + (long)b * p.Lcap;
    uint8_t* pb = protect + (long)b * p.Lcap;
    uint8_t* kb = keep + (long)b * p.Lcap;
    int32_t* hb = holes + (long)b * p.Lcap;
    int32_t* mvb = movers + (long)b * p.Lcap;

    if (n == 0) {
        if (tid == 0) { n_move[b] = 0; if (evicted_count) evicted_count[b] = 0; }
        return;
    }
    // per-head softmax statistics over the live entries: thread = (part, head)
    const int parts = blockDim.x / H;                // host guarantees H <= blockDim.x; threads beyond parts*H idle here
    const int h = tid % H, part = tid / H;
    {
        float mx = -INFINITY;
        if (part < parts)
            for (int j = part; j < n; j += parts) mx = fmaxf(mx, lb[(long)j * H + h]);
        if (part < parts) s_part[part * H + h] = mx;
        __syncthreads();
        if (tid < H) {
            float m2 = -INFINITY;
            for (int q = 0; q < parts; ++q) m2 = fmaxf(m2, s_part[q * H + tid]);
            s_max[tid] = m2;
        }
        __syncthreads();
        const float mh = s_max[h];
        float z = 0.f;
        if (part < parts)
            for (int j = part; j < n; j += parts) z += fast_exp2((lb[(long)j * H + h] - mh) * kLog2eD);
        if (part < parts) s_part[part * H + h] = z;
        __syncthreads();
        if (tid < H) {
            float z2 = 0.f;
            for (int q = 0; q < parts; ++q) z2 += s_part[q * H + tid];
            s_inv[tid] = 1.0f / (z2 * (float)H);
        }
        __syncthreads();
    }
    // a_t[j] = mean_h softmax ; acc <- decay*acc + a_t
    for (int j = tid; j < n; j += blockDim.x) {
        float a = 0.f;
        for (int hh = 0; hh < H; ++hh) a += fast_exp2((lb[(long)j * H + hh] - s_max[hh]) * kLog2eD) * s_inv[hh];
        ab[j] = fmaf(decay, ab[j], a);
    }
    __syncthreads();

    if (n <= budget) {                               // nothing to evict
        if (tid == 0) { n_move[b] = 0; if (evicted_count) evicted_count[b] = 0; }
        return;
    }
    int np = 0;
    for (int j = tid; j < n; j += blockDim.x) np += pb[j] != 0;
    np = block_sum_i(np, s_red);
    const int nu = n - np;
    const int extra = min(max(budget - np, 0), nu);
    const int new_len = np + extra;
    SelectBound sb{0ull, 63};
    if (extra > 0) {
        auto keyfn = [&](int i, bool& ok) -> uint64_t {
            ok = pb[i] == 0;
            return ok ? rank_key(ab[i], ib[i]) : 0ull;
        };
        sb = block_radix_select(keyfn, n, extra, s_hist);
    }
    // keep flags, hole / mover / evicted lists (ascending slot order by construction of the scan)
    int run_h = 0, run_m = 0, run_e = 0;
    for (int base = 0; base < n; base += blockDim.x) {
        const int j = base + tid;
        bool kp = false;
        if (j < n) {
            kp = pb[j] != 0 || (extra > 0 && (rank_key(ab[j], ib[j]) >> sb.shift) >= sb.bound);
            kb[j] = kp;
        }
        const bool is_hole = j < new_len && !kp;
        const bool is_mover = j >= new_len && j < n && kp;
        const bool is_ev = j < n && !kp;
        int th, tm, te;
        const int rh = block_rank(is_hole, s_red, th);
        const int rm = block_rank(is_mover, s_red, tm);
        const int re = block_rank(is_ev, s_red, te);
        if (is_hole) hb[run_h + rh] = j;
        if (is_mover) mvb[run_m + rm] = j;
        if (is_ev && evicted_ids) evicted_ids[(long)b * p.Lcap + run_e + re] = ib[j];
        run_h += th; run_m += tm; run_e += te;
    }
    __syncthreads();
    // move the small per-entry arrays (sources >= new_len, destinations < new_len: no overlap)
    for (int t = tid; t < run_m; t += blockDim.x) {
        const int src = mvb[t], dst = hb[t];
        ab[dst] = ab[src];
        ib[dst] = ib[src];
        pb[dst] = pb[src];
    }
    if (tid == 0) {
        n_move[b] = run_m;
        len[b] = new_len;
        if (evicted_count) evicted_count[b] = run_e;
    }
}

// The static policy (Sec. 3.5): the entries to keep are given, nothing is scored.  One block per
// sample turns the keep flags into the same hole / mover lists as the selection kernels and moves the
// small per-entry arrays; the row moves then run over every layer's cache.
__global__ __launch_bounds__(1024) void decode_keep_plan_kernel(
    DecodeDims p, const uint8_t* __restrict__ keep, float* __restrict__ acc, int32_t* __restrict__ ids,
    uint8_t* __restrict__ protect, int32_t* __restrict__ len,
    int32_t* __restrict__ holes, int32_t* __restrict__ movers, int32_t* __restrict__ n_move,
    int32_t* __restrict__ evicted_ids, int32_t* __restrict__ evicted_count)
{
    __shared__ int s_red[16];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = min(max(len[b], 0), p.Lcap);
    const uint8_t* kf = keep + (long)b * p.Lcap;
    float* ab = acc ? acc + (long)b * p.Lcap : nullptr;
    int32_t* ib = ids + (long)b * p.Lcap;
    uint8_t* pb = protect + (long)b * p.Lcap;
    int32_t* hb = holes + (long)b * p.Lcap;
    int32_t* mvb = movers + (long)b * p.Lcap;

    int nk = 0;
    for (int j = tid; j < n; j += blockDim.x) nk += kf[j] != 0;
    const int new_len = block_sum_i(nk, s_red);
    // hole / mover / evicted lists (ascending slot order by construction of the scan)
    int run_h = 0, run_m = 0, run_e = 0;
    for (int base = 0; base < n; base += blockDim.x) {
        const int j = base + tid;
        const bool kp = j < n && kf[j] != 0;
        const bool is_hole = j < new_len && !kp;
        const bool is_mover = j >= new_len && j < n && kp;
        const bool is_ev = j < n && !kp;
        int th, tm, te;
        const int rh = block_rank(is_hole, s_red, th);
        const int rm = block_rank(is_mover, s_red, tm);
        const int re = block_rank(is_ev, s_red, te);
        if (is_hole) hb[run_h + rh] = j;
        if (is_mover) mvb[run_m + rm] = j;
        if (is_ev && evicted_ids) evicted_ids[(long)b * p.Lcap + run_e + re] = ib[j];
        run_h += th; run_m += tm; run_e += te;
    }
    __syncthreads();
    // move the small per-entry arrays (sources >= new_len, destinations < new_len: no overlap)
    for (int t = tid; t < run_m; t += blockDim.x) {
        const int src = mvb[t], dst = hb[t];
        if (ab) ab[dst] = ab[src];
        ib[dst] = ib[src];
        pb[dst] = pb[src];
    }
    if (tid == 0) {
        n_move[b] = run_m;
        len[b] = new_len;
        if (evicted_count) evicted_count[b] = run_e;
    }
}

// Row moves: block (g, b, layer) copies movers[t] -> holes[t] for t = g, g + gridDim.x, ... in the
// cache of its layer (layer_stride 16-byte vectors apart; one layer for the per-step policy).
// STREAM_ONCE: caches too large to stay resident -- the source rows are dead after the move and the
// destination rows will not be read from cache either, so both sides bypass it.
template <bool STREAM_ONCE>
__global__ __launch_bounds__(256) void decode_move_kernel(
    DecodeDims p, const int32_t* __restrict__ holes, const int32_t* __restrict__ movers,
    const int32_t* __restrict__ n_move, u32x4* __restrict__ k_cache, u32x4* __restrict__ v_cache, long layer_stride)
{
    const int b = blockIdx.y;
    // the first pair of the lists is requested together with the count (the entry exists whatever the
    // count is; it is used only if the count says so)
    const int t0 = min((int)blockIdx.x, p.Lcap - 1);
    int mv = movers[(long)b * p.Lcap + t0], hl = holes[(long)b * p.Lcap + t0];
    const int nm = n_move[b];
    const int rv = p.H * p.d / 8;
    k_cache += blockIdx.z * layer_stride;
    v_cache += blockIdx.z * layer_stride;
    // source rows (beyond the new length) and destination rows (holes below it) never coincide, but
    // the compiler cannot know: the vectors of a round are read into registers before any is written
    for (int t = blockIdx.x; t < nm; t += gridDim.x) {
        const long src = ((long)b * p.Lcap + mv) * rv;
        const long dst = ((long)b * p.Lcap + hl) * rv;
        const int tn = min(t + (int)gridDim.x, p.Lcap - 1);                  // next pair, in flight during the copy
        mv = movers[(long)b * p.Lcap + tn];
        hl = holes[(long)b * p.Lcap + tn];
        for (int c = threadIdx.x; c < rv; c += 2 * blockDim.x) {
            const int c2 = c + blockDim.x;
            const bool two = c2 < rv;
            auto ld = [](const u32x4* q) { return STREAM_ONCE ? __builtin_nontemporal_load(q) : *q; };
            auto st = [](u32x4* q, const u32x4& v) { if (STREAM_ONCE) __builtin_nontemporal_store(v, q); else *q = v; };
            // the V rows are not read on this path at all (only moved): always streamed
            const u32x4 k0 = ld(k_cache + src + c), v0 = __builtin_nontemporal_load(v_cache + src + c);
            u32x4 k1 = k0, v1 = v0;
            if (two) { k1 = ld(k_cache + src + c2); v1 = __builtin_nontemporal_load(v_cache + src + c2); }
            st(k_cache + dst + c, k0);
            __builtin_nontemporal_store(v0, v_cache + dst + c);
            if (two) { st(k_cache + dst + c2, k1); __builtin_nontemporal_store(v1, v_cache + dst + c2); }
        }
    }
}

__global__ __launch_bounds__(256) void decode_append_kernel(
    DecodeDims p, const u32x4* __restrict__ k_new, const u32x4* __restrict__ v_new,
    u32x4* __restrict__ k_cache, u32x4* __restrict__ v_cache,
    float* __restrict__ acc, int32_t* __restrict__ ids, uint8_t* __restrict__ protect, int32_t* __restrict__ len,
    int32_t new_id, int protect_new)
{
    const int b = blockIdx.x;
    const int slot = len[b];
    if (slot < 0 || slot >= p.Lcap) return;
    const int rv = p.H * p.d / 8;
    const long dst = ((long)b * p.Lcap + slot) * rv;
    for (int c = threadIdx.x; c < rv; c += blockDim.x) {
        k_cache[dst + c] = k_new[(long)b * rv + c];
        v_cache[dst + c] = v_new[(long)b * rv + c];
    }
    __syncthreads();                                   // every thread has read len[b] before it changes
    if (threadIdx.x == 0) {
        acc[(long)b * p.Lcap + slot] = 0.f;
        ids[(long)b * p.Lcap + slot] = new_id;
        protect[(long)b * p.Lcap + slot] = protect_new ? 1 : 0;
        len[b] = slot + 1;
    }
}

// The two kernels above for caches in other layouts: a row is walked head slice by head slice.
__global__ __launch_bounds__(256) void decode_move_strided_kernel(
    DecodeDims p, KvLayout lay, const int32_t* __restrict__ holes, const int32_t* __restrict__ movers,
    const int32_t* __restrict__ n_move, uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache, long layer_stride)
{
    const int b = blockIdx.y;
    const int nm = n_move[b];
    const int lph = p.d / 8, rv = p.H * lph;
    k_cache += blockIdx.z * layer_stride + (long)b * lay.batch;
    v_cache += blockIdx.z * layer_stride + (long)b * lay.batch;
    for (int t = blockIdx.x; t < nm; t += gridDim.x) {
        const long src = (long)movers[(long)b * p.Lcap + t] * lay.token;
        const long dst = (long)holes[(long)b * p.Lcap + t] * lay.token;
        for (int c = threadIdx.x; c < rv; c += blockDim.x) {
            const int h = c / lph, w = c - h * lph;
            const long off = (long)h * lay.head + w * 8;
            const u32x4 k0 = *reinterpret_cast<const u32x4*>(k_cache + src + off);
            const u32x4 v0 = *reinterpret_cast<const u32x4*>(v_cache + src + off);
            *reinterpret_cast<u32x4*>(k_cache + dst + off) = k0;
            *reinterpret_cast<u32x4*>(v_cache + dst + off) = v0;
        }
    }
}

__global__ __launch_bounds__(256) void decode_append_strided_kernel(
    DecodeDims p, KvLayout lay, const u32x4* __restrict__ k_new, const u32x4* __restrict__ v_new,
    uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache,
    float* __restrict__ acc, int32_t* __restrict__ ids, uint8_t* __restrict__ protect, int32_t* __restrict__ len,
    int32_t new_id, int protect_new)
{
    const int b = blockIdx.x;
    const int slot = len[b];
    if (slot < 0 || slot >= p.Lcap) return;
    const int lph = p.d / 8, rv = p.H * lph;
    const long dst = (long)b * lay.batch + (long)slot * lay.token;
    for (int c = threadIdx.x; c < rv; c += blockDim.x) {
        const int h = c / lph, w = c - h * lph;
        const long off = dst + (long)h * lay.head + w * 8;
        *reinterpret_cast<u32x4*>(k_cache + off) = k_new[(long)b * rv + c];
        *reinterpret_cast<u32x4*>(v_cache + off) = v_new[(long)b * rv + c];
    }
    __syncthreads();                                   // every thread has read len[b] before it changes
    if (threadIdx.x == 0) {
        acc[(long)b * p.Lcap + slot] = 0.f;
        ids[(long)b * p.Lcap + slot] = new_id;
        protect[(long)b * p.Lcap + slot] = protect_new ? 1 : 0;
        len[b] = slot + 1;
    }
}

#ifndef MD_DEC_BLOCKS
#define MD_DEC_BLOCKS 4096   // target number of blocks of the streaming logits kernel
#endif

struct DecodeWorkspace {
    float* logits; float2* stat_partial; uint8_t* keep; int32_t* holes; int32_t* movers; int32_t* n_move;
    size_t bytes;
};

DecodeWorkspace carve_decode(void* base, int B, int Lcap, int H) {
    Carver c(base);
    DecodeWorkspace w;
    w.logits = c.take<float>((size_t)B * Lcap * H);
    w.stat_partial = c.take<float2>((size_t)B * kMaxStatParts * H);
    w.keep = c.take<uint8_t>((size_t)B * Lcap);
    w.holes = c.take<int32_t>((size_t)B * Lcap);
    w.movers = c.take<int32_t>((size_t)B * Lcap);
    w.n_move = c.take<int32_t>((size_t)B);
    w.bytes = c.off;
    return w;
}

int check_decode_dims(const char* who, int B, int Lcap, int H, int d) {
    if (B <= 0 || Lcap <= 0 || H <= 0 || d <= 0) return fail(MD_EINVAL, "%s: B, Lcap, H, d must be positive", who);
    if (d != 8 && d != 16 && d != 32 && d != 64 && d != 128 && d != 256 && d != 512)
        return fail(MD_ESHAPE, "%s: head dim %d must be a power of two in [8, 512]", who, d);
    if (H > 1024) return fail(MD_ESHAPE, "%s: H=%d exceeds the limit of 1024 heads", who, H);
    if ((long)B * Lcap > (1l << 28)) return fail(MD_ESHAPE, "%s: cache too large", who);
    return MD_OK;
}

}  // namespace
}  // namespace md

using namespace md;


extern "C" size_t mustdrop_decode_evict_workspace_bytes(int B, int Lcap, int H) {
    if (B <= 0 || Lcap <= 0 || H <= 0) return 0;
    return carve_decode(nullptr, B, Lcap, H).bytes;
}

namespace md {
namespace {

int decode_evict_impl(
    const void* q, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d,
    float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count,
    const md_kv_layout* cache_layout,
    void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    int rc = check_decode_dims("decode_evict", B, Lcap, H, d);
    if (rc != MD_OK) return rc;
    KvLayout lay;
    rc = read_layout("decode_evict", "cache", cache_layout, B, Lcap, H, d, &lay);
    if (rc != MD_OK) return rc;
    const bool dense = is_dense(lay, Lcap, H, d);
    if (!q || !k_cache || !v_cache || !acc || !ids || !protect || !len)
        return fail(MD_EINVAL, "decode_evict: q, the caches and the state arrays are required");
    if (budget < 0) return fail(MD_EINVAL, "decode_evict: negative budget");
    if (std::isnan(softmax_scale) || std::isnan(decay)) return fail(MD_EINVAL, "decode_evict: NaN parameter");
    // the selection ranks entries by the bit pattern of their running score, which orders non-negative values only
    if (decay < 0.f) return fail(MD_EINVAL, "decode_evict: decay must be >= 0 (running scores stay non-negative)");
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache))
        return fail(MD_EALIGN, "decode_evict: q and the caches must be 16-byte aligned");
    const size_t cache_bytes = layout_extent_bytes(lay, B, Lcap, H, d);
    if (overlaps(k_cache, cache_bytes, v_cache, cache_bytes)) return fail(MD_EALIAS, "decode_evict: k_cache overlaps v_cache");
    if (overlaps(q, (size_t)B * H * d * 2, k_cache, cache_bytes) || overlaps(q, (size_t)B * H * d * 2, v_cache, cache_bytes))
        return fail(MD_EALIAS, "decode_evict: q overlaps a cache");
    const DecodeWorkspace w = carve_decode(workspace, B, Lcap, H);
    {
        // the small state arrays, the optional outputs and the workspace against the caches, q and one another
        const size_t n = (size_t)B * Lcap;
        const void* pa[] = {acc, ids, protect, len, evicted_ids, evicted_count, workspace, k_cache, v_cache, q};
        const size_t sa[] = {n * 4, n * 4, n, (size_t)B * 4, n * 4, (size_t)B * 4, workspace ? w.bytes : 0,
                             cache_bytes, cache_bytes, (size_t)B * H * d * 2};
        for (int a = 0; a < 7; ++a)
            for (int c = a + 1; c < 10; ++c)
                if (overlaps(pa[a], sa[a], pa[c], sa[c]))
                    return fail(MD_EALIAS, "decode_evict: the state arrays, outputs, workspace, caches and q must not overlap");
    }
    if (!workspace || workspace_bytes < w.bytes)
        return fail(MD_EWORKSPACE, "decode_evict: workspace of %zu bytes needed, %zu given", w.bytes, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(MD_EALIGN, "decode_evict: workspace must be 256-byte aligned");

    DecodeDims p{B, Lcap, H, d};
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint16_t* qp = static_cast<const uint16_t*>(q);
    const uint16_t* kp = static_cast<const uint16_t*>(k_cache);
    const int row_bytes = H * d * 2;
    const int nit = row_bytes % 1024 == 0 ? row_bytes / 1024 : 0;
    int n_part = 0;                                   // > 0: the logits kernel left per-block softmax statistics
    if (d == 128 && (nit == 1 || nit == 2 || nit == 4 || nit == 8)) {
        // streaming shape: about 16 waves per CU in flight, each striding over its sample's entries
        int blocks_x = (MD_DEC_BLOCKS + B - 1) / B;
        const int max_x = (Lcap + 3) / 4;
        if (blocks_x > max_x) blocks_x = max_x;
        if (blocks_x > kMaxStatParts) blocks_x = kMaxStatParts;
        if (blocks_x < 1) blocks_x = 1;
        dim3 g1(blocks_x, B);
#define MD_STREAM2(NIT_, S_, O_)                                                                                   \
        MD_LAUNCH("decode_logits", st, (decode_logits_stream_kernel<16, NIT_, S_, O_>), g1, 256, 0,                \
            qp, kp, len, p, lay, softmax_scale, w.logits, w.stat_partial)
#define MD_STREAM(NIT_, S_) do { if (stream_once) MD_STREAM2(NIT_, S_, true); else MD_STREAM2(NIT_, S_, false); } while (0)
        // a cache beyond half of the 256 MB Infinity Cache is streamed; a smaller one is kept cached for
        // the row moves that follow
        const bool stream_once = cache_bytes > (size_t)128 << 20;
        if (dense) {
            switch (nit) {
                case 1: MD_STREAM(1, false); break;
                case 2: MD_STREAM(2, false); break;
                case 4: MD_STREAM(4, false); break;
                default: MD_STREAM(8, false); break;
            }
        } else {
            switch (nit) {
                case 1: MD_STREAM(1, true); break;
                case 2: MD_STREAM(2, true); break;
                case 4: MD_STREAM(4, true); break;
                default: MD_STREAM(8, true); break;
            }
        }
#undef MD_STREAM2
#undef MD_STREAM
        n_part = blocks_x;
    } else {
        int tpb = (int)(((long)B * Lcap + 4095) / 4096);
        tpb = tpb < 4 ? 4 : (tpb > 32 ? 32 : tpb);
        dim3 g1((Lcap + tpb - 1) / tpb, B);
        switch (d / 8) {
            case 1: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<1>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            case 2: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<2>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            case 4: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<4>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            case 8: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<8>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            case 16: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<16>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            case 32: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<32>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
            default: MD_LAUNCH("decode_logits", st, (decode_logits_kernel<64>), g1, 256, 0, qp, kp, len, p, lay, softmax_scale, tpb, w.logits); break;
        }
    }
    const bool fast_h = H == 4 || H == 8 || H == 16 || H == 32 || H == 64;
    if (n_part > 0 && Lcap <= 8192 && fast_h) {
        const size_t lds = 2 * sizeof(int) * (size_t)Lcap;
        const int ipt = (Lcap + 1023) / 1024;
#define MD_SELECT_FAST(I, E)                                                                                       \
    MD_LAUNCH("decode_select", st, (decode_select_fast_kernel<I, E>), B, 1024, lds,                          \
        p, w.logits, w.stat_partial, n_part, decay, budget, acc, ids, protect, len, w.holes, w.movers, w.n_move,   \
        evicted_ids, evicted_count)
#define MD_SELECT_FAST_H(I)                                                                                        \
    switch (H) {                                                                                                   \
        case 4: MD_SELECT_FAST(I, 1); break;                                                                       \
        case 8: MD_SELECT_FAST(I, 2); break;                                                                       \
        case 16: MD_SELECT_FAST(I, 4); break;                                                                      \
        case 32: MD_SELECT_FAST(I, 8); break;                                                                      \
        default: MD_SELECT_FAST(I, 16); break;                                                                     \
    }
        if (ipt <= 1) { MD_SELECT_FAST_H(1) }
        else if (ipt <= 2) { MD_SELECT_FAST_H(2) }
        else if (ipt <= 3) { MD_SELECT_FAST_H(3) }
        else if (ipt <= 4) { MD_SELECT_FAST_H(4) }
        else if (ipt <= 5) { MD_SELECT_FAST_H(5) }
        else if (ipt <= 6) { MD_SELECT_FAST_H(6) }
        else { MD_SELECT_FAST_H(8) }
#undef MD_SELECT_FAST_H
#undef MD_SELECT_FAST
    } else {
        const size_t lds = sizeof(float) * ((size_t)2 * H + 1024);
        MD_LAUNCH("decode_select", st, (decode_select_kernel), B, 1024, lds,
            p, w.logits, decay, budget, acc, ids, protect, len, w.keep, w.holes, w.movers, w.n_move, evicted_ids, evicted_count);
    }
    // blocks per sample: enough that a small batch still covers the chip and a block has one or two rows to move
    const int move_x = B >= 32 ? 32 : (B >= 16 ? 64 : 128);
    dim3 g3(move_x, B);
    if (dense && cache_bytes > (size_t)128 << 20)
        MD_LAUNCH("decode_move", st, (decode_move_kernel<true>), g3, 256, 0,
            p, w.holes, w.movers, w.n_move, static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache), 0l);
    else if (dense)
        MD_LAUNCH("decode_move", st, (decode_move_kernel<false>), g3, 256, 0,
            p, w.holes, w.movers, w.n_move, static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache), 0l);
    else
        MD_LAUNCH("decode_move", st, (decode_move_strided_kernel), g3, 256, 0,
            p, lay, w.holes, w.movers, w.n_move, static_cast<uint16_t*>(k_cache), static_cast<uint16_t*>(v_cache), 0l);
    return check_launch("decode_evict");
}

int decode_keep_impl(
    void* k_cache, void* v_cache, const uint8_t* keep,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d,
    int32_t* evicted_ids, int32_t* evicted_count,
    const md_kv_layout* cache_layout, int64_t layer_stride_in,
    void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    int rc = check_decode_dims("decode_keep", B, Lcap, H, d);
    if (rc != MD_OK) return rc;
    if (n_layers <= 0 || n_layers > 65535) return fail(MD_EINVAL, "decode_keep: n_layers=%d out of range", n_layers);
    KvLayout lay;
    rc = read_layout("decode_keep", "cache", cache_layout, B, Lcap, H, d, &lay);
    if (rc != MD_OK) return rc;
    const size_t layer_bytes = layout_extent_bytes(lay, B, Lcap, H, d);
    long layer_stride = cache_layout ? (long)layer_stride_in : (long)B * Lcap * H * d;
    if (n_layers == 1) layer_stride = (long)(layer_bytes / 2);
    if (layer_stride <= 0 || layer_stride % 8 || (size_t)layer_stride * 2 < layer_bytes)
        return fail(MD_ESHAPE, "decode_keep: layer_stride=%ld must be a multiple of 8 elements covering one layer (%zu elements)",
                    layer_stride, layer_bytes / 2);
    const bool dense = is_dense(lay, Lcap, H, d);
    if (!k_cache || !v_cache || !keep || !ids || !protect || !len)
        return fail(MD_EINVAL, "decode_keep: null pointer among the required arguments");
    if ((H * d * 2) % 16) return fail(MD_EALIGN, "decode_keep: a row of H*d=%d bf16 is not a multiple of 16 bytes", H * d);
    if (!aligned16(k_cache) || !aligned16(v_cache)) return fail(MD_EALIGN, "decode_keep: caches must be 16-byte aligned");
    const size_t cache_bytes = (size_t)(n_layers - 1) * layer_stride * 2 + layer_bytes;
    if (overlaps(k_cache, cache_bytes, v_cache, cache_bytes)) return fail(MD_EALIAS, "decode_keep: k_cache overlaps v_cache");
    const DecodeWorkspace w = carve_decode(workspace, B, Lcap, H);
    if (!workspace || workspace_bytes < w.bytes)
        return fail(MD_EWORKSPACE, "decode_keep: workspace of %zu bytes needed, %zu given", w.bytes, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(MD_EALIGN, "decode_keep: workspace must be 256-byte aligned");

    DecodeDims p{B, Lcap, H, d};
    hipStream_t st = static_cast<hipStream_t>(stream);
    MD_LAUNCH("decode_keep_plan", st, (decode_keep_plan_kernel), B, 1024, 0,
        p, keep, acc, ids, protect, len, w.holes, w.movers, w.n_move, evicted_ids, evicted_count);
    dim3 g3(32, B, n_layers);
    if (dense && cache_bytes > (size_t)128 << 20)
        MD_LAUNCH("decode_move", st, (decode_move_kernel<true>), g3, 256, 0,
            p, w.holes, w.movers, w.n_move, static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache),
            layer_stride / 8);
    else if (dense)
        MD_LAUNCH("decode_move", st, (decode_move_kernel<false>), g3, 256, 0,
            p, w.holes, w.movers, w.n_move, static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache),
            layer_stride / 8);
    else
        MD_LAUNCH("decode_move", st, (decode_move_strided_kernel), g3, 256, 0,
            p, lay, w.holes, w.movers, w.n_move, static_cast<uint16_t*>(k_cache), static_cast<uint16_t*>(v_cache),
            layer_stride);
    return check_launch("decode_keep");
}

int decode_append_impl(
    const void* k_new, const void* v_new, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, int32_t new_id, int protect_new, const md_kv_layout* cache_layout, void* stream)
{
    clear_error();
    int rc = check_decode_dims("decode_append", B, Lcap, H, d);
    if (rc != MD_OK) return rc;
    KvLayout lay;
    rc = read_layout("decode_append", "cache", cache_layout, B, Lcap, H, d, &lay);
    if (rc != MD_OK) return rc;
    if (!k_new || !v_new || !k_cache || !v_cache || !acc || !ids || !protect || !len)
        return fail(MD_EINVAL, "decode_append: all pointers are required");
    if (new_id < 0) return fail(MD_EINVAL, "decode_append: ids must be non-negative");
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return fail(MD_EALIGN, "decode_append: tensors must be 16-byte aligned");
    DecodeDims p{B, Lcap, H, d};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (is_dense(lay, Lcap, H, d))
        MD_LAUNCH("decode_append", st, (decode_append_kernel), B, 256, 0,
            p, static_cast<const u32x4*>(k_new), static_cast<const u32x4*>(v_new),
            static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache), acc, ids, protect, len, new_id, protect_new);
    else
        MD_LAUNCH("decode_append", st, (decode_append_strided_kernel), B, 256, 0,
            p, lay, static_cast<const u32x4*>(k_new), static_cast<const u32x4*>(v_new),
            static_cast<uint16_t*>(k_cache), static_cast<uint16_t*>(v_cache), acc, ids, protect, len, new_id, protect_new);
    return check_launch("decode_append");
}

}  // namespace
}  // namespace md

extern "C" int mustdrop_decode_evict(
    const void* q, void* k_cache, void* v_cache, float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_evict_impl(q, k_cache, v_cache, acc, ids, protect, len, B, Lcap, H, d, softmax_scale, decay, budget,
                             evicted_ids, evicted_count, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_decode_evict_strided(
    const void* q, void* k_cache, void* v_cache, float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count, const md_kv_layout* cache_layout,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_evict_impl(q, k_cache, v_cache, acc, ids, protect, len, B, Lcap, H, d, softmax_scale, decay, budget,
                             evicted_ids, evicted_count, cache_layout, workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_decode_keep(
    void* k_cache, void* v_cache, const uint8_t* keep, float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d, int32_t* evicted_ids, int32_t* evicted_count,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_keep_impl(k_cache, v_cache, keep, acc, ids, protect, len, n_layers, B, Lcap, H, d, evicted_ids,
                            evicted_count, nullptr, 0, workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_decode_keep_strided(
    void* k_cache, void* v_cache, const uint8_t* keep, float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d, int32_t* evicted_ids, int32_t* evicted_count,
    const md_kv_layout* cache_layout, int64_t layer_stride, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_keep_impl(k_cache, v_cache, keep, acc, ids, protect, len, n_layers, B, Lcap, H, d, evicted_ids,
                            evicted_count, cache_layout, layer_stride, workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_decode_append(
    const void* k_new, const void* v_new, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, int32_t new_id, int protect_new, void* stream)
{
    return decode_append_impl(k_new, v_new, k_cache, v_cache, acc, ids, protect, len, B, Lcap, H, d, new_id, protect_new,
                              nullptr, stream);
}

extern "C" int mustdrop_decode_append_strided(
    const void* k_new, const void* v_new, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, int32_t new_id, int protect_new, const md_kv_layout* cache_layout, void* stream)
{
    return decode_append_impl(k_new, v_new, k_cache, v_cache, acc, ids, protect, len, B, Lcap, H, d, new_id, protect_new,
                              cache_layout, stream);
}
