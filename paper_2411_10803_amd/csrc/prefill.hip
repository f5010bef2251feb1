// Stage 2 -- prefill (Sec. 3.4): text-to-vision attention scores, the dual filter (Eq. 8-10) and
// token drop (stable compaction of hidden states, K and V).
//
// The column statistics V_j = sum_i a_ij and I_j = max_i a_ij need the row softmax normaliser of
// every text row over the WHOLE key axis, and the head mean has to be taken before the max over
// text rows.  So the scores take two sweeps over K:
//   prefill_rowstats_kernel  per (sample, head, key chunk): S = K Q^T on the MFMA units, online
//                            (max, sum-exp) per text row -> partial row statistics
//   prefill_colscore_kernel  per (sample, 32 vision keys): waves split the heads, recompute S,
//                            p = exp(s - m)/Z, accumulate the head mean in registers, reduce the
//                            waves through LDS in a fixed order, column sum / max -> V_j, I_j
// The N x Mv probability matrix is never written to memory.
//   prefill_select_kernel    per sample: G, the filter rule (threshold) or radix top-k (budget),
//                            prefix sum -> kept_index, row map for the copy
//   prefill_compact_kernel   one block per output row: 16-byte vector copies of hidden, K, V rows
//
// MFMA tile: v_mfma_f32_32x32x16_bf16, keys on the M side (A operand), text rows on the N side
// (B operand).  In the result a lane holds one text row (column lane%32) and 16 of the 32 keys,
// so the row-softmax reductions over keys stay inside a lane (+ one exchange with lane^32).
#include "md_device.hpp"
#include "md_host.hpp"

namespace md {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct PrefillDims {
    int B, Mv, N, H, d, C, L;
    int nch;          // key chunks per (sample, head) in the row-statistics sweep
    int chunk;        // keys per chunk (multiple of 32)
    int Npad;         // 32 * NB
    int Rcap;
};

// key row of accumulator register r in the 32x32 result tile
__device__ __forceinline__ int tile_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// A 32-row operand tile (32 keys or 32 text rows of one head, 16*KS bf16 each) on its way from
// global memory to MFMA fragments.  Global loads are coalesced: a row's head slice is CH = 2*KS
// consecutive 16-byte chunks, 64/CH rows per load instruction.  The tile is then written to a
// wave-private LDS buffer (row pitch padded by 16 bytes: conflict-free 128-bit reads) and read back
// in fragment layout: lane (g = lane/32, r = lane%32) holds row r, chunks 2*ks+g, ks = 0..KS-1.
template <int KS>
struct OperandTile {
    static constexpr int CH = 2 * KS;
    static constexpr int ROWS_PER_LOAD = kWave / CH;
    static constexpr int PITCH = CH * 16 + 16;
    static constexpr int BYTES = 32 * PITCH;

    // rows row0..row0+31 of a matrix whose rows are `row_stride` elements apart; rows >= nrows read as zero
    __device__ static __forceinline__ void gload(const uint16_t* base, long row_stride, int row0, int nrows, int lane,
                                                 u32x4 (&st)[KS]) {
        const int chunk = lane % CH, sub = lane / CH;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int r = row0 + t * ROWS_PER_LOAD + sub;
            if (r < nrows) st[t] = *reinterpret_cast<const u32x4*>(base + (long)r * row_stride + chunk * 8);
            else st[t] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    __device__ static __forceinline__ void to_lds(char* tile, int lane, const u32x4 (&st)[KS]) {
        const int chunk = lane % CH, sub = lane / CH;
#pragma unroll
        for (int t = 0; t < KS; ++t)
            *reinterpret_cast<u32x4*>(tile + (t * ROWS_PER_LOAD + sub) * PITCH + chunk * 16) = st[t];
    }
    __device__ static __forceinline__ void frags(const char* tile, int lane, bf16x8 (&f)[KS]) {
        const char* p = tile + (lane & 31) * PITCH + (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(p + ks * 32);
    }
};

// LDS traffic between lanes of one wave: LDS operations of a wave execute in order, the fence keeps
// the compiler from moving the reads above the writes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------------------------
// Sweep 1: row statistics.  Block = (key chunk, head, sample), 4 waves; every wave walks its share
// of the chunk's 32-key tiles with the next tile's global loads in flight during the MFMAs.
// Chunk 0 also stores the text-query fragments in fragment-major order (qfrag) so that sweep 2
// reads them with fully coalesced 16-byte loads.
template <int NB, int KS>
__global__ __launch_bounds__(256) void prefill_rowstats_kernel(
    const uint16_t* __restrict__ q_txt, const uint16_t* __restrict__ k,
    const uint8_t* __restrict__ vis_valid, PrefillDims p, float scale_log2e,
    float2* __restrict__ partial, bf16x8* __restrict__ qfrag)
{
    using Tile = OperandTile<KS>;
    __shared__ __attribute__((aligned(16))) char s_tile[4][Tile::BYTES];
    __shared__ float s_m[4][32 * NB], s_z[4][32 * NB];
    const int lane = lane_id(), wv = wave_id();
    const int ch = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const long tok_stride = (long)p.H * p.d;
    const uint16_t* kb = k + ((long)b * p.L * p.H + h) * p.d;
    const uint16_t* qb = q_txt + ((long)b * p.N * p.H + h) * p.d;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * p.Mv : nullptr;
    char* tile = s_tile[wv];

    const int c0 = ch * p.chunk;
    const int c1 = min(c0 + p.chunk, p.L);
    int j0 = c0 + 32 * wv;
    u32x4 st[KS];
    if (j0 < c1) Tile::gload(kb, tok_stride, j0, p.L, lane, st);

    // text-query fragments of this head: through the same LDS tile, one 32-row block at a time
    bf16x8 qf[NB][KS];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        u32x4 sq[KS];
        Tile::gload(qb, tok_stride, 32 * nb, p.N, lane, sq);
        Tile::to_lds(tile, lane, sq);
        wave_lds_sync();
        Tile::frags(tile, lane, qf[nb]);
        wave_lds_sync();
        if (ch == 0 && wv == 0) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qfrag[((((long)b * p.H + h) * NB + nb) * KS + ks) * kWave + lane] = qf[nb][ks];
        }
    }

    float m[NB], z[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { m[nb] = -INFINITY; z[nb] = 0.f; }

    for (; j0 < c1; j0 += 32 * 4) {
        Tile::to_lds(tile, lane, st);
        wave_lds_sync();
        bf16x8 kf[KS];
        Tile::frags(tile, lane, kf);
        wave_lds_sync();
        if (j0 + 32 * 4 < c1) Tile::gload(kb, tok_stride, j0 + 32 * 4, p.L, lane, st);   // prefetch
        // validity of the 32 keys of this tile as a bit mask (vision keys only)
        const int jl = j0 + (lane & 31);
        const bool v_ok = jl < p.Mv ? (!vb || vb[jl]) : false;
        const uint32_t vmask = (uint32_t)__ballot(v_ok);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[nb][ks], acc, 0, 0, 0);
            const int i = 32 * nb + (lane & 31);
            float t[16];
            float bm = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile_row(r, lane);
                const int j = j0 + row;
                const bool vis = j < p.Mv ? ((vmask >> row) & 1u) : (j < p.L && (j - p.Mv) <= i);
                t[r] = vis ? acc[r] * scale_log2e : -INFINITY;
                bm = fmaxf(bm, t[r]);
            }
            const float mn = fmaxf(m[nb], bm);
            if (mn > -INFINITY) {
                float s = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) s += exp2f(t[r] - mn);
                z[nb] = z[nb] * exp2f(m[nb] - mn) + s;
                m[nb] = mn;
            }
        }
    }
    // merge the two lane halves (same text row, the other 16 keys), then the four waves
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float mo = __shfl_xor(m[nb], 32, kWave), zo = __shfl_xor(z[nb], 32, kWave);
        const float mn = fmaxf(m[nb], mo);
        float zn = 0.f;
        if (mn > -INFINITY) zn = z[nb] * exp2f(m[nb] - mn) + zo * exp2f(mo - mn);
        if (lane < 32) { s_m[wv][32 * nb + lane] = mn; s_z[wv][32 * nb + lane] = zn; }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * NB; i += blockDim.x) {
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, s_m[w][i]);
        float zn = 0.f;
        if (mn > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) zn += s_z[w][i] * exp2f(s_m[w][i] - mn);
        }
        partial[(((long)b * p.H + h) * p.nch + ch) * p.Npad + i] = make_float2(mn, zn);
    }
}

// ---------------------------------------------------------------------------------------------
// Sweep 2: column scores.  Block = (tile of 32*MB vision keys, sample), NW waves; wave w takes heads
// w, w+NW, ...  K tiles go global -> registers (prefetched one head ahead) -> wave-private LDS ->
// fragments; text-query fragments come from qfrag with coalesced loads.
template <int NB, int KS, int NW, int MB>
__global__ __launch_bounds__(64 * NW) void prefill_colscore_kernel(
    const bf16x8* __restrict__ qfrag, const uint16_t* __restrict__ k,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len,
    const float2* __restrict__ partial, PrefillDims p, float scale_log2e,
    float* __restrict__ Vout, float* __restrict__ Iout)
{
    using Tile = OperandTile<KS>;
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    constexpr int NP = 32 * NB, TJ = 32 * MB, PARTS = 2 * NW;
    char* s_tiles = smem_raw;                                                   // [NW][MB][Tile::BYTES]
    float* s_m = reinterpret_cast<float*>(smem_raw + NW * MB * Tile::BYTES);    // [H][NP] row max (log2 domain)
    float* s_iz = s_m + p.H * NP;            // [H][NP]  1 / (Z * H)
    float* s_a = s_iz + p.H * NP;            // [TJ][NP + 1] head-mean probabilities of this key tile
    float* s_ps = s_a + TJ * (NP + 1);       // [PARTS][TJ] partial column sums
    float* s_pm = s_ps + PARTS * TJ;         // [PARTS][TJ] partial column maxima

    const int lane = lane_id(), wv = wave_id(), tid = threadIdx.x;
    const int j0 = blockIdx.x * TJ, b = blockIdx.y;
    const long tok_stride = (long)p.H * p.d;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * p.Mv : nullptr;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    char* tile = s_tiles + wv * MB * Tile::BYTES;

    // first head's K tiles are requested before anything else
    u32x4 st[MB][KS];
    {
        const uint16_t* kb = k + ((long)b * p.L * p.H + wv) * p.d;
        if (wv < p.H) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) Tile::gload(kb, tok_stride, j0 + 32 * mb, p.Mv, lane, st[mb]);
        }
    }

    // combine the chunk partials into the row statistics of every (head, text row) of this sample
    const float inv_h = 1.0f / (float)p.H;
    for (int e = tid; e < p.H * NP; e += blockDim.x) {
        const int h = e / NP, i = e % NP;
        const float2* pp = partial + ((long)b * p.H + h) * p.nch * p.Npad + i;
        float mn = -INFINITY, zn = 0.f;
        for (int c = 0; c < p.nch; ++c) {
            const float2 v = pp[(long)c * p.Npad];
            const float m2 = fmaxf(mn, v.x);
            if (m2 > -INFINITY) zn = zn * exp2f(mn - m2) + v.y * exp2f(v.x - m2);
            mn = m2;
        }
        s_m[e] = mn;
        s_iz[e] = zn > 0.f ? inv_h / zn : 0.f;
    }
    __syncthreads();

    f32x16 a_acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) a_acc[mb][nb][r] = 0.f;

    for (int h = wv; h < p.H; h += NW) {
        bf16x8 kf[MB][KS];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) Tile::to_lds(tile + mb * Tile::BYTES, lane, st[mb]);
        wave_lds_sync();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) Tile::frags(tile + mb * Tile::BYTES, lane, kf[mb]);
        wave_lds_sync();
        if (h + NW < p.H) {                                                     // prefetch the next head's K tiles
            const uint16_t* kb = k + ((long)b * p.L * p.H + (h + NW)) * p.d;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) Tile::gload(kb, tok_stride, j0 + 32 * mb, p.Mv, lane, st[mb]);
        }
        const bf16x8* qh = qfrag + ((long)b * p.H + h) * NB * KS * kWave + lane;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            bf16x8 qf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[ks] = qh[(nb * KS + ks) * kWave];
            const int i = 32 * nb + (lane & 31);
            const float mi = s_m[h * NP + i], izi = s_iz[h * NP + i];
            const bool row_ok = i < tl;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                f32x16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mb][ks], qf[ks], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // masking by select: padded rows / keys may hold NaN
                    const float pr = row_ok ? exp2f(acc[r] * scale_log2e - mi) * izi : 0.f;
                    a_acc[mb][nb][r] += pr;
                }
            }
        }
    }

    // sum the waves' head groups in wave order (fixed order -> reproducible bits)
    for (int w = 0; w < NW; ++w) {
        if (wv == w) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float* cell = &s_a[(32 * mb + tile_row(r, lane)) * (NP + 1) + 32 * nb + (lane & 31)];
                        if (w == 0) *cell = a_acc[mb][nb][r];
                        else *cell += a_acc[mb][nb][r];
                    }
        }
        __syncthreads();
    }
    // Eq. 8 / Eq. 10: column sum and column max over the text rows
    for (int e = tid; e < PARTS * TJ; e += blockDim.x) {
        const int r = e % TJ, part = e / TJ;
        const int per = (NP + PARTS - 1) / PARTS;
        float s = 0.f, mx = 0.f;
        for (int i = part * per; i < min((part + 1) * per, tl); ++i) {
            const float a = s_a[r * (NP + 1) + i];
            s += a;
            mx = fmaxf(mx, a);
        }
        s_ps[e] = s;
        s_pm[e] = mx;
    }
    __syncthreads();
    if (tid < TJ) {
        const int j = j0 + tid;
        if (j < p.Mv) {
            float s = 0.f, mx = 0.f;
            for (int part = 0; part < PARTS; ++part) { s += s_ps[part * TJ + tid]; mx = fmaxf(mx, s_pm[part * TJ + tid]); }
            const bool ok = !vb || vb[j];
            Vout[(long)b * p.Mv + j] = ok ? s : 0.f;
            Iout[(long)b * p.Mv + j] = ok ? mx : 0.f;
        }
    }
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void prefill_select_kernel(
    PrefillDims p, const float* __restrict__ V, const float* __restrict__ I,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len, const uint8_t* __restrict__ is_key,
    int mode, int budget, float gamma, float alpha,
    float* __restrict__ score, int32_t* __restrict__ src_row,
    int32_t* __restrict__ kept_index, int32_t* __restrict__ kept_count,
    int32_t* __restrict__ out_len, uint8_t* __restrict__ out_protect,
    float* __restrict__ score_global, float* __restrict__ score_indiv)
{
    __shared__ float s_redf[16];
    __shared__ int s_red[16];
    __shared__ int s_hist[256];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int Mv = p.Mv;
    const float* Vb = V + (long)b * Mv;
    const float* Ib = I + (long)b * Mv;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * Mv : nullptr;
    const uint8_t* kb = is_key ? is_key + (long)b * Mv : nullptr;
    float* sc = score + (long)b * Mv;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    const int rows_cap = p.Rcap + p.N;

    // G = sum of V_j over valid vision tokens (Eq. 9, right-hand side); fixed summation tree
    float part = 0.f;
    for (int j = tid; j < Mv; j += blockDim.x) {
        const float v = Vb[j];
        part += v;                                   // invalid tokens carry 0
        if (score_global) score_global[(long)b * Mv + j] = v;
        if (score_indiv) score_indiv[(long)b * Mv + j] = Ib[j];
    }
    const float G = block_sum(part, s_redf);

    SelectBound sb{0ull, 63};
    int extra = 0;
    if (mode == MD_FILTER_BUDGET) {
        int nk = 0, no = 0;
        const float gG = gamma * G;
        for (int j = tid; j < Mv; j += blockDim.x) {
            const bool ok = !vb || vb[j];
            const bool key = ok && kb && kb[j];
            nk += key;
            no += ok && !key;
            const float s1 = G > 0.f ? Vb[j] / gG : 0.f;
            const float s2 = Ib[j] / alpha;
            sc[j] = fmaxf(s1, s2);
        }
        nk = block_sum_i(nk, s_red);
        no = block_sum_i(no, s_red);
        extra = min(max(budget - nk, 0), no);
        __syncthreads();
        if (extra > 0) {
            auto keyfn = [&](int i, bool& ok) -> uint64_t {
                ok = (!vb || vb[i]) && !(kb && kb[i]);
                return ok ? rank_key(sc[i], i) : 0ull;
            };
            sb = block_radix_select(keyfn, Mv, extra, s_hist);
        }
    }
    const float thrV = gamma * G;

    int running = 0;
    for (int base = 0; base < Mv; base += blockDim.x) {
        const int j = base + tid;
        bool keep = false, key = false;
        if (j < Mv && (!vb || vb[j])) {
            key = kb && kb[j];
            if (mode == MD_FILTER_THRESHOLD) {
                const bool drop = (Vb[j] <= thrV) && (Ib[j] < alpha) && !key;
                keep = !drop;
            } else {
                keep = key || (extra > 0 && (rank_key(sc[j], j) >> sb.shift) >= sb.bound);
            }
        }
        int total;
        const int r = block_rank(keep, s_red, total);
        const int o = running + r;
        if (keep && o < p.Rcap) {
            kept_index[(long)b * p.Rcap + o] = j;
            src_row[(long)b * rows_cap + o] = j;
            if (out_protect) out_protect[(long)b * rows_cap + o] = key ? 1 : 0;
        }
        running += total;
    }
    const int nkept = min(running, p.Rcap);
    for (int i = tid; i < rows_cap - nkept; i += blockDim.x) {
        const int o = nkept + i;
        src_row[(long)b * rows_cap + o] = i < tl ? Mv + i : -1;
        if (out_protect && i < tl) out_protect[(long)b * rows_cap + o] = 1;
    }
    if (tid == 0) {
        kept_count[b] = running;
        if (out_len) out_len[b] = nkept + tl;
    }
}

// One block per output row: copies the hidden, K and V rows named by the row map.
__global__ __launch_bounds__(256) void prefill_compact_kernel(
    PrefillDims p, const int32_t* __restrict__ src_row,
    const u32x4* __restrict__ hidden, const u32x4* __restrict__ k, const u32x4* __restrict__ v,
    u32x4* __restrict__ hidden_out, u32x4* __restrict__ k_out, u32x4* __restrict__ v_out)
{
    const int o = blockIdx.x, b = blockIdx.y;
    const int rows_cap = p.Rcap + p.N;
    const int src = src_row[(long)b * rows_cap + o];
    if (src < 0) return;
    const int hv = p.C / 8, kv = p.H * p.d / 8;          // 16-byte vectors per row
    const u32x4* hs = hidden + ((long)b * p.L + src) * hv;
    const u32x4* ks = k + ((long)b * p.L + src) * kv;
    const u32x4* vs = v + ((long)b * p.L + src) * kv;
    u32x4* hd = hidden_out + ((long)b * rows_cap + o) * hv;
    u32x4* kd = k_out + ((long)b * rows_cap + o) * kv;
    u32x4* vd = v_out + ((long)b * rows_cap + o) * kv;
    for (int c = threadIdx.x; c < hv; c += blockDim.x) hd[c] = hs[c];
    for (int c = threadIdx.x; c < kv; c += blockDim.x) { kd[c] = ks[c]; vd[c] = vs[c]; }
}

struct PrefillWorkspace {
    float2* partial; bf16x8* qfrag; float* V; float* I; float* score; int32_t* src_row;
    size_t bytes;
};

#ifndef MD_PF_NW
#define MD_PF_NW 4      // waves per block in the column-score sweep
#endif
#ifndef MD_PF_MB
#define MD_PF_MB 1      // 32-key tiles per block in the column-score sweep
#endif

int pick_chunks(int B, int H, int L) {
    // enough (sample, head, chunk) blocks to cover the 256 CUs several times; chunks of whole tiles
    // about two resident blocks per CU (512 in all); at least 4 tiles per chunk so every wave has work
    const int tiles = (L + 31) / 32;
    int nch = (512 + B * H - 1) / (B * H);
    if (nch > tiles / 4) nch = tiles / 4;
    if (nch < 1) nch = 1;
    if (nch > 64) nch = 64;
    return nch;
}

PrefillWorkspace carve_prefill(void* base, int B, int Mv, int N, int H, int Rcap) {
    Carver c(base);
    PrefillWorkspace w;
    const int Npad = (N + 31) / 32 * 32;
    w.partial = c.take<float2>((size_t)B * H * 64 * Npad);
    w.qfrag = c.take<bf16x8>((size_t)B * H * Npad * 16);      // [B][H][NB][KS][64] fragments, d <= 128
    w.V = c.take<float>((size_t)B * Mv);
    w.I = c.take<float>((size_t)B * Mv);
    w.score = c.take<float>((size_t)B * Mv);
    w.src_row = c.take<int32_t>((size_t)B * (Rcap + N));
    w.bytes = c.off;
    return w;
}

template <int NB, int KS>
int launch_scores(const PrefillDims& p, const PrefillWorkspace& w, hipStream_t st, const void* q_txt, const void* k,
                  const uint8_t* vis_valid, const int32_t* txt_len, float scale_log2e) {
    constexpr int NW = MD_PF_NW, MB = MD_PF_MB, TJ = 32 * MB;
    dim3 g1(p.nch, p.H, p.B);
    MD_LAUNCH("prefill_rowstats", st, (prefill_rowstats_kernel<NB, KS><<<g1, 256, 0, st>>>(
        static_cast<const uint16_t*>(q_txt), static_cast<const uint16_t*>(k), vis_valid, p, scale_log2e, w.partial,
        w.qfrag)));
    const size_t lds = (size_t)NW * MB * OperandTile<KS>::BYTES +
                       sizeof(float) * ((size_t)2 * p.H * 32 * NB + TJ * (32 * NB + 1) + 2 * (2 * NW * TJ));
    auto kern = prefill_colscore_kernel<NB, KS, NW, MB>;
    static bool attr_set = false;             // per template instance: raise the dynamic-LDS limit once
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return fail(MD_EHIP, "prefill_filter: cannot raise the LDS limit: %s", hipGetErrorString(e));
        attr_set = true;
    }
    if (lds > 160 * 1024) return fail(MD_ESHAPE, "prefill_filter: H=%d, N=%d need %zu bytes of LDS (limit 160 KiB)", p.H, p.N, lds);
    dim3 g2((p.Mv + TJ - 1) / TJ, p.B);
    MD_LAUNCH("prefill_colscore", st, (kern<<<g2, 64 * NW, lds, st>>>(
        w.qfrag, static_cast<const uint16_t*>(k), vis_valid, txt_len, w.partial, p, scale_log2e, w.V, w.I)));
    return MD_OK;
}

}  // namespace
}  // namespace md

using namespace md;

extern "C" size_t mustdrop_prefill_filter_workspace_bytes(int B, int Mv, int N, int H, int Rcap) {
    if (B <= 0 || Mv <= 0 || N <= 0 || H <= 0 || Rcap <= 0) return 0;
    return carve_prefill(nullptr, B, Mv, N, H, Rcap).bytes;
}

extern "C" int mustdrop_prefill_filter(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    if (mode != MD_FILTER_BUDGET && mode != MD_FILTER_THRESHOLD) return fail(MD_EDTYPE, "prefill_filter: unknown mode %d", (int)mode);
    if (B <= 0 || Mv <= 0 || N <= 0 || H <= 0 || d <= 0 || C <= 0 || Rcap <= 0)
        return fail(MD_EINVAL, "prefill_filter: B, Mv, N, H, d, C, Rcap must be positive");
    if (!q_txt || !k || !v || !hidden || !hidden_out || !k_out || !v_out || !kept_index || !kept_count)
        return fail(MD_EINVAL, "prefill_filter: q_txt, k, v, hidden, the *_out tensors, kept_index and kept_count are required");
    if (d != 64 && d != 128) return fail(MD_ESHAPE, "prefill_filter: head dim %d not supported (64 or 128)", d);
    if (N > 128) return fail(MD_ESHAPE, "prefill_filter: N=%d text tokens exceeds the limit of 128", N);
    if (H > 128) return fail(MD_ESHAPE, "prefill_filter: H=%d heads exceeds the limit of 128", H);
    if ((long)B * (Mv + N) > (1l << 28)) return fail(MD_ESHAPE, "prefill_filter: too many tokens");
    if (C % 8) return fail(MD_EALIGN, "prefill_filter: a hidden row of C=%d bf16 is not a multiple of 16 bytes", C);
    if (std::isnan(softmax_scale) || std::isnan(gamma) || std::isnan(alpha)) return fail(MD_EINVAL, "prefill_filter: NaN parameter");
    if (mode == MD_FILTER_BUDGET) {
        if (budget < 0) return fail(MD_EINVAL, "prefill_filter: negative budget");
        if (!(gamma > 0.f) || !(alpha > 0.f)) return fail(MD_EINVAL, "prefill_filter: budget mode needs gamma > 0 and alpha > 0");
        if (Rcap < (budget < Mv ? budget : Mv))
            return fail(MD_EINVAL, "prefill_filter: Rcap=%d is smaller than min(budget, Mv)=%d", Rcap, budget < Mv ? budget : Mv);
    }
    const void* big[] = {q_txt, k, v, hidden, hidden_out, k_out, v_out};
    for (const void* ptr : big)
        if (!aligned16(ptr)) return fail(MD_EALIGN, "prefill_filter: tensor pointers must be 16-byte aligned");
    const size_t L = (size_t)Mv + N;
    const size_t kv_in = (size_t)B * L * H * d * 2, h_in = (size_t)B * L * C * 2;
    const size_t kv_out = (size_t)B * (Rcap + N) * H * d * 2, h_out = (size_t)B * (Rcap + N) * C * 2;
    const void* ins[] = {k, v, hidden, q_txt};
    const size_t in_sz[] = {kv_in, kv_in, h_in, (size_t)B * N * H * d * 2};
    const void* outs[] = {k_out, v_out, hidden_out};
    const size_t out_sz[] = {kv_out, kv_out, h_out};
    for (int a = 0; a < 3; ++a)
        for (int c = 0; c < 4; ++c)
            if (overlaps(outs[a], out_sz[a], ins[c], in_sz[c])) return fail(MD_EALIAS, "prefill_filter: an output tensor overlaps an input");
    const PrefillWorkspace w = carve_prefill(workspace, B, Mv, N, H, Rcap);
    if (!workspace || workspace_bytes < w.bytes)
        return fail(MD_EWORKSPACE, "prefill_filter: workspace of %zu bytes needed, %zu given", w.bytes, workspace ? workspace_bytes : (size_t)0);
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(MD_EALIGN, "prefill_filter: workspace must be 256-byte aligned");

    PrefillDims p;
    p.B = B; p.Mv = Mv; p.N = N; p.H = H; p.d = d; p.C = C; p.L = Mv + N; p.Rcap = Rcap;
    p.Npad = (N + 31) / 32 * 32;
    p.nch = pick_chunks(B, H, p.L);
    const int tiles = (p.L + 31) / 32;
    p.chunk = (tiles + p.nch - 1) / p.nch * 32;
    p.nch = (p.L + p.chunk - 1) / p.chunk;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float sl2 = softmax_scale * kLog2e;

    int rc = MD_OK;
    const int NB = p.Npad / 32;
    if (d == 128) {
        if (NB == 1) rc = launch_scores<1, 8>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else if (NB == 2) rc = launch_scores<2, 8>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else if (NB == 3) rc = launch_scores<3, 8>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else rc = launch_scores<4, 8>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
    } else {
        if (NB == 1) rc = launch_scores<1, 4>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else if (NB == 2) rc = launch_scores<2, 4>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else if (NB == 3) rc = launch_scores<3, 4>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
        else rc = launch_scores<4, 4>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
    }
    if (rc != MD_OK) return rc;
    int32_t* src_row = out_ids ? out_ids : w.src_row;     // the row map doubles as the optional out_ids
    MD_LAUNCH("prefill_select", st, (prefill_select_kernel<<<B, 1024, 0, st>>>(
        p, w.V, w.I, vis_valid, txt_len, is_key, (int)mode, budget, gamma, alpha,
        w.score, src_row, kept_index, kept_count, out_len, out_protect, score_global, score_indiv)));
    dim3 gc(Rcap + N, B);
    MD_LAUNCH("prefill_compact", st, (prefill_compact_kernel<<<gc, 256, 0, st>>>(p, src_row,
        static_cast<const u32x4*>(hidden), static_cast<const u32x4*>(k), static_cast<const u32x4*>(v),
        static_cast<u32x4*>(hidden_out), static_cast<u32x4*>(k_out), static_cast<u32x4*>(v_out))));
    return check_launch("prefill_filter");
}
