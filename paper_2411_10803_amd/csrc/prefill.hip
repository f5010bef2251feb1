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
    KvLayout q, kv;   // element strides of q_txt and of k (v shares them)
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
    // The same for a tile whose 32 rows all exist.  tile_base: first row of the tile (wave-uniform),
    // lane_off: from lane_offset(); the addresses are a scalar base plus a tile-invariant lane offset,
    // so a load costs no vector arithmetic.
    __device__ static __forceinline__ uint32_t lane_offset(long row_stride, int lane) {
        return (uint32_t)(((lane / CH) * row_stride + (lane % CH) * 8) * 2);
    }
    __device__ static __forceinline__ void gload_full(const uint16_t* tile_base, long row_stride, uint32_t lane_off,
                                                      u32x4 (&st)[KS]) {
#pragma unroll
        for (int t = 0; t < KS; ++t)
            st[t] = *reinterpret_cast<const u32x4*>(
                reinterpret_cast<const char*>(tile_base + (long)t * ROWS_PER_LOAD * row_stride) + lane_off);
    }
    // either of the two, by a wave-uniform test
    __device__ static __forceinline__ void gload_any(const uint16_t* base, long row_stride, int row0, int nrows, int lane,
                                                     uint32_t lane_off, u32x4 (&st)[KS]) {
        if (row0 + 32 <= nrows) gload_full(base + (long)row0 * row_stride, row_stride, lane_off, st);
        else gload(base, row_stride, row0, nrows, lane, st);
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

// Row statistics folded into one constant: a probability of the head mean is
// exp2(s*scale*log2e + c) with c = -m - log2(Z) - log2(H); text rows beyond txt_len get -inf (-> 0).
__device__ __forceinline__ float fold_stats(float m, float z, bool row_ok, int H) {
    return (row_ok && z > 0.f) ? -m - fast_log2(z) - fast_log2((float)H) : -INFINITY;
}

// LDS traffic between lanes of one wave: LDS operations of a wave execute in order, the fence keeps
// the compiler from moving the reads above the writes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------------------------
// Sweep 1: row statistics.  Block = (key chunk x text group, head, sample), 4 waves; every wave
// walks its share of the chunk's 32-key tiles with the next tile's global loads in flight during
// the MFMAs.  A block covers NB <= 2 blocks of 32 text rows (one "text group"); longer prompts are
// split over blockIdx.x.  Chunk 0 also stores the text-query fragments in fragment-major order
// (qfrag), rows beyond txt_len zeroed, so that sweep 2 reads them with coalesced 16-byte loads.
template <int NB, int KS>
__global__ __launch_bounds__(256) void prefill_rowstats_kernel(
    const uint16_t* __restrict__ q_txt, const uint16_t* __restrict__ k,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len, PrefillDims p, float scale_log2e,
    float2* __restrict__ partial, float* __restrict__ cstat, bf16x8* __restrict__ qfrag)
{
    using Tile = OperandTile<KS>;
    __shared__ __attribute__((aligned(16))) char s_tile[4][Tile::BYTES];
    __shared__ float s_m[4][32 * NB], s_z[4][32 * NB];
    const int lane = lane_id(), wv = wave_id();
    // Blocks go round-robin over the 8 XCDs in launch order.  With several text groups, the blocks that
    // read the same K chunk (same chunk and head, different text group) are placed 8 apart in that order:
    // same XCD, launched together, so the second reader finds the chunk in that XCD's L2.
    int ch = blockIdx.x % p.nch, tg = blockIdx.x / p.nch, h = blockIdx.y;
    const int b = blockIdx.z;
    const int ntg = gridDim.x / p.nch;
    if (ntg > 1 && (p.nch * p.H) % 8 == 0) {
        const int lin = blockIdx.x + gridDim.x * blockIdx.y;
        const int r = lin % (8 * ntg), pair = lin / (8 * ntg) * 8 + r % 8;
        tg = r / 8;
        ch = pair % p.nch;
        h = pair / p.nch;
    }
    const int i_base = tg * 32 * NB;                 // first text row of this block's group
    const long tok_stride = p.kv.token;
    const uint16_t* kb = k + (long)b * p.kv.batch + (long)h * p.kv.head;
    const uint16_t* qb = q_txt + (long)b * p.q.batch + (long)h * p.q.head;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * p.Mv : nullptr;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    char* tile = s_tile[wv];

    const int c0 = ch * p.chunk;
    const int c1 = min(c0 + p.chunk, p.L);
    int j0 = c0 + 32 * wv;
    u32x4 st[KS];
    // validity of this lane's key (lane % 32) in the tile that is in flight; fetched with the tile so
    // that its latency hides behind the previous tile's arithmetic
    // (kept as the loaded byte until the next iteration: turning it into a lane mask right away would
    // make the wave wait for the load, and with it for the tile that was requested just before)
    auto key_valid = [&](int j) -> uint32_t {
        const int jl = j + (lane & 31);
        return vb ? (uint32_t)vb[min(jl, p.Mv - 1)] : 1u;
    };
    uint32_t v_nxt = 0;
    const uint32_t lane_off = Tile::lane_offset(tok_stride, lane);
    if (j0 < c1) {
        Tile::gload_any(kb, tok_stride, j0, p.L, lane, lane_off, st);
        v_nxt = key_valid(j0);
    }

    // text-query fragments of this head: through the same LDS tile, one 32-row block at a time
    // (all loads are issued before the first LDS pass: the fences below would otherwise serialise them)
    bf16x8 qf[NB][KS];
    constexpr int NST = NB < 2 ? NB : 2;             // text blocks staged at a time (32 registers each)
#pragma unroll
    for (int nb0 = 0; nb0 < NB; nb0 += NST) {
        u32x4 sq[NST][KS];
#pragma unroll
        for (int e = 0; e < NST; ++e)
            Tile::gload(qb, p.q.token, i_base + 32 * (nb0 + e), tl, lane, sq[e]);   // rows >= txt_len read as zero
#pragma unroll
        for (int e = 0; e < NST; ++e) {
            const int nb = nb0 + e;
            Tile::to_lds(tile, lane, sq[e]);
            wave_lds_sync();
            Tile::frags(tile, lane, qf[nb]);
            wave_lds_sync();
            const int nbg = tg * NB + nb;            // 32-row block index within the padded text axis
            if (ch == 0 && wv == 0 && nbg < p.Npad / 32) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    qfrag[((((long)b * p.H + h) * (p.Npad / 32) + nbg) * KS + ks) * kWave + lane] = qf[nb][ks];
            }
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
        const bool v_ok = v_nxt != 0 && j0 + (lane & 31) < p.Mv;
        if (j0 + 32 * 4 < c1) {                                                 // prefetch
            Tile::gload_any(kb, tok_stride, j0 + 32 * 4, p.L, lane, lane_off, st);
            v_nxt = key_valid(j0 + 32 * 4);
        }
        // validity of the 32 keys of this tile as a bit mask (vision keys only)
        const uint32_t vmask = (uint32_t)__ballot(v_ok);
        // three wave-uniform cases: a vision tile without holes, a vision tile with dropped keys,
        // and a tile that reaches into the text keys (causal mask, per text row)
        const bool vision_tile = j0 + 32 <= p.Mv;
        const bool all_visible = vision_tile && vmask == 0xFFFFFFFFu;
        const uint32_t mine = vmask >> (4 * (lane >> 5));   // tile_row(r, lane) = 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[nb][ks], acc, 0, 0, 0);
            // invisible entries become -inf; the positive scale is applied after the maximum
            float bm = -INFINITY;
            if (all_visible) {
#pragma unroll
                for (int r = 0; r < 16; ++r) bm = fmaxf(bm, acc[r]);
            } else if (vision_tile) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    if (!((mine >> (8 * (r >> 2) + (r & 3))) & 1u)) acc[r] = -INFINITY;
                    bm = fmaxf(bm, acc[r]);
                }
            } else {
                const int i = i_base + 32 * nb + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = tile_row(r, lane);
                    const int j = j0 + row;
                    const bool vis = j < p.Mv ? ((vmask >> row) & 1u) : (j < p.L && (j - p.Mv) <= i);
                    if (!vis) acc[r] = -INFINITY;
                    bm = fmaxf(bm, acc[r]);
                }
            }
            const float mn = fmaxf(m[nb], bm * scale_log2e);
            if (mn > -INFINITY) {
                float s = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) s += fast_exp2(fmaf(acc[r], scale_log2e, -mn));
                z[nb] = z[nb] * fast_exp2(m[nb] - mn) + s;
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
        if (mn > -INFINITY) zn = z[nb] * fast_exp2(m[nb] - mn) + zo * fast_exp2(mo - mn);
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
            for (int w = 0; w < 4; ++w) zn += s_z[w][i] * fast_exp2(s_m[w][i] - mn);
        }
        if (i_base + i < p.Npad) {
            if (p.nch == 1)     // the only chunk: fold the statistics right away (see fold_stats)
                cstat[((long)b * p.H + h) * p.Npad + i_base + i] = fold_stats(mn, zn, i_base + i < tl, p.H);
            else
                partial[(((long)b * p.H + h) * p.nch + ch) * p.Npad + i_base + i] = make_float2(mn, zn);
        }
    }
}

// Several key chunks per (sample, head): merge their partial statistics.  One thread per text row.
__global__ __launch_bounds__(256) void prefill_cstat_kernel(
    const float2* __restrict__ partial, const int32_t* __restrict__ txt_len, PrefillDims p, float* __restrict__ cstat)
{
    const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (long)p.B * p.H * p.Npad) return;
    const int i = (int)(e % p.Npad);
    const long bh = e / p.Npad;
    const int b = (int)(bh / p.H);
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    const float2* pp = partial + bh * p.nch * p.Npad + i;
    float mn = -INFINITY, zn = 0.f;
    for (int c = 0; c < p.nch; ++c) {
        const float2 v = pp[(long)c * p.Npad];
        const float m2 = fmaxf(mn, v.x);
        if (m2 > -INFINITY) zn = zn * fast_exp2(mn - m2) + v.y * fast_exp2(v.x - m2);
        mn = m2;
    }
    cstat[e] = fold_stats(mn, zn, i < tl, p.H);
}

// ---------------------------------------------------------------------------------------------
// Sweep 2: column scores.  Block = (32 vision keys, sample), NW waves; wave w takes heads w, w+NW, ...
// K tiles go global -> registers (prefetched one head ahead) -> wave-private LDS -> fragments;
// text-query fragments come from qfrag with coalesced loads.  The row statistics are folded into one
// constant per (head, text row): p = exp2(s*scale*log2e + c), c = -m - log2(Z*H), so a probability
// costs one FMA and one exp2.  NB <= 4 = number of 32-row text blocks of this launch, starting at
// block nb0: prompts of more than 128 rows take one launch per 128 rows, each writing its own
// partial column sums and maxima, merged by prefill_merge_groups_kernel.
template <int NB, int KS, int NW>
__global__ __launch_bounds__(64 * NW) void prefill_colscore_kernel(
    const bf16x8* __restrict__ qfrag, const uint16_t* __restrict__ k,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len,
    const float* __restrict__ cstat, PrefillDims p, float scale_log2e, int nb0,
    float* __restrict__ Vout, float* __restrict__ Iout)
{
    using Tile = OperandTile<KS>;
    constexpr int PARTS = 2 * NW;
    constexpr int HALF = NB > 2 ? 2 : NB;            // text blocks dumped per reduction round (8 KiB per wave)
    static_assert(32 * 32 * HALF * 4 <= Tile::BYTES || KS < 8, "reduction buffer must fit the K tile");
    constexpr int WBUF = (Tile::BYTES > 32 * 32 * HALF * 4) ? Tile::BYTES : 32 * 32 * HALF * 4;
    __shared__ __attribute__((aligned(16))) char s_buf[NW][WBUF];   // K tile of each wave; later its a_acc dump
    __shared__ float s_ps[PARTS][32], s_pm[PARTS][32];

    const int lane = lane_id(), wv = wave_id(), tid = threadIdx.x;
    // Workgroups go round-robin over the 8 XCDs (each with its own L2).  All key tiles of a sample
    // share that sample's query fragments, so a sample is pinned to one XCD when the batch allows:
    // its fragments are then fetched into one L2 instead of eight.
    const int nt = (p.Mv + 31) / 32;
    int b, tile_idx;
    if (p.B % 8 == 0) {
        const int xcd = blockIdx.x % 8, r = blockIdx.x / 8;
        b = xcd + 8 * (r / nt);
        tile_idx = r % nt;
    } else if (8 % p.B == 0) {                       // small batch: a sample owns 8/B XCDs
        const int g = 8 / p.B, xcd = blockIdx.x % 8, r = blockIdx.x / 8;
        b = xcd / g;
        tile_idx = r * g + xcd % g;
        if (tile_idx >= nt) return;                  // grid padded to a multiple of 8 (whole block leaves)
    } else {
        b = blockIdx.x / nt;
        tile_idx = blockIdx.x % nt;
    }
    const int j0 = tile_idx * 32;
    const long tok_stride = p.kv.token;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * p.Mv : nullptr;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    char* tile = s_buf[wv];

    u32x4 st[KS];
    const uint16_t* kb = k + (long)b * p.kv.batch;
    if (wv < p.H) Tile::gload(kb + (long)wv * p.kv.head, tok_stride, j0, p.Mv, lane, st);

    f32x16 a_acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a_acc[nb][r] = 0.f;

    constexpr int TP = (NB + 1) / 2;                 // text blocks are processed in pairs (64 registers of fragments)
    for (int h = wv; h < p.H; h += NW) {
        const bf16x8* qh = qfrag + (((long)b * p.H + h) * (p.Npad / 32) + nb0) * KS * kWave + lane;
        const float* ch = cstat + ((long)b * p.H + h) * p.Npad + 32 * nb0 + (lane & 31);
        bf16x8 qf[2][KS];
        float c[2];
        auto load_pair = [&](int tp) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int nb = 2 * tp + e;
                if (nb < NB) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) qf[e][ks] = qh[(nb * KS + ks) * kWave];
                    c[e] = ch[32 * nb];
                }
            }
        };
        // the first pair's query fragments and folded row statistics are requested before the K tile
        // goes through LDS, so they are in flight meanwhile
        load_pair(0);
        bf16x8 kf[KS];
        Tile::to_lds(tile, lane, st);
        wave_lds_sync();
        Tile::frags(tile, lane, kf);
        wave_lds_sync();
        if (h + NW < p.H)                                                      // prefetch the next head's K tile
            Tile::gload(kb + (long)(h + NW) * p.kv.head, tok_stride, j0, p.Mv, lane, st);
#pragma unroll
        for (int tp = 0; tp < TP; ++tp) {
            if (tp > 0) load_pair(tp);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int nb = 2 * tp + e;
                if (nb < NB) {
                    f32x16 acc;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[e][ks], acc, 0, 0, 0);
                    // text rows beyond txt_len have zero query fragments and c = -inf: exp2(-inf) = 0 exactly
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        a_acc[nb < NB ? nb : 0][r] += fast_exp2(fmaf(acc[r], scale_log2e, c[e]));
                }
            }
        }
    }

    // Column statistics (Eq. 8 / Eq. 10).  Every wave dumps its accumulators into its own buffer;
    // the waves' head groups are then summed in wave order while the text rows are reduced
    // (fixed order -> reproducible bits).
    float col_s = 0.f, col_m = 0.f;                  // this thread's (key, text-row slice) partial results
    const int rr = tid & 31, part = tid >> 5;
#pragma unroll
    for (int half = 0; half < NB; half += HALF) {
        __syncthreads();
        float* mine = reinterpret_cast<float*>(tile);
#pragma unroll
        for (int nb = 0; nb < HALF; ++nb) {
            if (half + nb < NB) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    mine[((nb * 32) + (lane & 31)) * 32 + ((tile_row(r, lane) + (lane & 31)) & 31)] =
                        a_acc[(half + nb) < NB ? (half + nb) : 0][r];
            }
        }
        __syncthreads();
        constexpr int per = (32 * HALF + PARTS - 1) / PARTS;
        for (int ii = part * per; ii < min((part + 1) * per, 32 * HALF); ++ii) {
            if ((nb0 + half) * 32 + ii >= tl) break;
            float a = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w)
                a += reinterpret_cast<const float*>(s_buf[w])[ii * 32 + ((rr + (ii & 31)) & 31)];
            col_s += a;
            col_m = fmaxf(col_m, a);
        }
    }
    s_ps[part][rr] = col_s;
    s_pm[part][rr] = col_m;
    __syncthreads();
    if (tid < 32) {
        const int j = j0 + tid;
        if (j < p.Mv) {
            float s = 0.f, mx = 0.f;
#pragma unroll
            for (int q = 0; q < PARTS; ++q) { s += s_ps[q][tid]; mx = fmaxf(mx, s_pm[q][tid]); }
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

// The same selection with a sample's scores held in registers (Mv <= 1024*IPT): tokens are dealt
// round-robin (thread t owns t, t+1024, ...), every global load is issued up front, the radix passes
// and the prefix sums touch no memory.
// The text rows of the outputs need no selection: in budget mode their place follows from counting the
// valid and the key tokens.  While the one block per sample of the selection kernel works through its
// dependent steps on 1 CU in 16, further blocks of the same launch copy those rows (hidden, K, V).
struct TextRows {
    const u32x4* hidden; const u32x4* k; const u32x4* v;
    u32x4* hidden_out; u32x4* k_out; u32x4* v_out;
    int enabled;
};
constexpr int kTextRowsPerBlock = 4;                 // 1024 threads = four rows of 256 threads

template <int IPT>
__device__ __forceinline__ void copy_text_rows(
    const PrefillDims& p, const TextRows& tr, const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len,
    const uint8_t* __restrict__ is_key, int budget, int* s_red)
{
    const int tid = threadIdx.x, Mv = p.Mv;
    const int bps = (p.N + kTextRowsPerBlock - 1) / kTextRowsPerBlock;        // blocks per sample
    const int e = blockIdx.x - p.B, b = e / bps, i = (e % bps) * kTextRowsPerBlock + tid / 256;
    // the number of vision rows kept, exactly as the selection block of this sample counts it
    uint32_t vv[IPT], kk[IPT];
#pragma unroll
    for (int t = 0; t < IPT; ++t) vv[t] = vis_valid ? vis_valid[(long)b * Mv + min(tid + t * 1024, Mv - 1)] : 1u;
#pragma unroll
    for (int t = 0; t < IPT; ++t) kk[t] = is_key ? is_key[(long)b * Mv + min(tid + t * 1024, Mv - 1)] : 0u;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    int cnt = 0;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        const bool ok = tid + t * 1024 < Mv && vv[t] != 0;
        cnt += (ok && kk[t] != 0 ? 1 : 0) + ((ok && kk[t] == 0) ? 1 << 16 : 0);
    }
    cnt = block_sum_i(cnt, s_red);
    const int nk = cnt & 0xFFFF, no = cnt >> 16;
    const int nkept = min(nk + min(max(budget - nk, 0), no), p.Rcap);
    if (i >= tl) return;
    const int rows_cap = p.Rcap + p.N;
    const int hv = p.C / 8, kv = p.H * p.d / 8, c0 = tid % 256;
    const long src = (long)b * p.L + Mv + i, dst = (long)b * rows_cap + nkept + i;
    for (int c = c0; c < kv; c += 256) {
        const u32x4 a = __builtin_nontemporal_load(tr.k + src * kv + c), a2 = __builtin_nontemporal_load(tr.v + src * kv + c);
        tr.k_out[dst * kv + c] = a;
        tr.v_out[dst * kv + c] = a2;
    }
    for (int c = c0; c < hv; c += 256) tr.hidden_out[dst * hv + c] = __builtin_nontemporal_load(tr.hidden + src * hv + c);
}

template <int IPT>
__global__ __launch_bounds__(1024) void prefill_select_fast_kernel(
    PrefillDims p, const float* __restrict__ V, const float* __restrict__ I,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len, const uint8_t* __restrict__ is_key,
    int mode, int budget, float gamma, float alpha,
    int32_t* __restrict__ src_row,
    int32_t* __restrict__ kept_index, int32_t* __restrict__ kept_count,
    int32_t* __restrict__ out_len, uint8_t* __restrict__ out_protect,
    float* __restrict__ score_global, float* __restrict__ score_indiv, TextRows tr)
{
    __shared__ float s_redf[16];
    __shared__ int s_red[16];
    __shared__ int s_hist[256];
    if ((int)blockIdx.x >= p.B) {                    // block-uniform: the blocks that copy the text rows
        copy_text_rows<IPT>(p, tr, vis_valid, txt_len, is_key, budget, s_red);
        return;
    }
    const int b = blockIdx.x, tid = threadIdx.x;
    const int Mv = p.Mv;
    const int rows_cap = p.Rcap + p.N;
    float v[IPT], iv[IPT];
    bool ok[IPT], key[IPT];
    {
        // every load at a clamped address and none guarded by another's result: one round trip
        uint32_t vv[IPT], kk[IPT];
#pragma unroll
        for (int t = 0; t < IPT; ++t) v[t] = V[(long)b * Mv + min(tid + t * 1024, Mv - 1)];
#pragma unroll
        for (int t = 0; t < IPT; ++t) iv[t] = I[(long)b * Mv + min(tid + t * 1024, Mv - 1)];
#pragma unroll
        for (int t = 0; t < IPT; ++t) vv[t] = vis_valid ? vis_valid[(long)b * Mv + min(tid + t * 1024, Mv - 1)] : 1u;
#pragma unroll
        for (int t = 0; t < IPT; ++t) kk[t] = is_key ? is_key[(long)b * Mv + min(tid + t * 1024, Mv - 1)] : 0u;
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const bool in = tid + t * 1024 < Mv;
            if (!in) { v[t] = 0.f; iv[t] = 0.f; }
            ok[t] = in && vv[t] != 0;
            key[t] = ok[t] && kk[t] != 0;
        }
    }
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    // G = sum of V_j over valid vision tokens (Eq. 9, right-hand side); fixed summation tree
    float part = 0.f;
    int cnt = 0;                                     // keys in the low half, other valid tokens in the high half
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        part += v[t];                                // invalid tokens carry 0
        cnt += (key[t] ? 1 : 0) + ((ok[t] && !key[t]) ? 1 << 16 : 0);
        const int j = tid + t * 1024;
        if (j < Mv) {
            if (score_global) score_global[(long)b * Mv + j] = v[t];
            if (score_indiv) score_indiv[(long)b * Mv + j] = iv[t];
        }
    }
    const float G = block_sum(part, s_redf);
    bool keep[IPT];
    if (mode == MD_FILTER_BUDGET) {
        cnt = block_sum_i(cnt, s_red);
        const int nk = cnt & 0xFFFF, no = cnt >> 16;
        const int extra = min(max(budget - nk, 0), no);
        const float gG = gamma * G;
        uint64_t rk[IPT];
#pragma unroll
        for (int t = 0; t < IPT; ++t) {
            const float s1 = G > 0.f ? v[t] / gG : 0.f;
            const float s2 = iv[t] / alpha;
            rk[t] = (ok[t] && !key[t]) ? rank_key(fmaxf(s1, s2), tid + t * 1024) : 0ull;
        }
        const SelectBound sb = block_radix_select_reg<IPT>(rk, extra, s_hist);
#pragma unroll
        for (int t = 0; t < IPT; ++t) keep[t] = key[t] || (rk[t] != 0 && extra > 0 && (rk[t] >> sb.shift) >= sb.bound);
    } else {
        const float thrV = gamma * G;
#pragma unroll
        for (int t = 0; t < IPT; ++t) keep[t] = ok[t] && !((v[t] <= thrV) && (iv[t] < alpha) && !key[t]);
    }
    int running = 0;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
        if (t * 1024 >= Mv) continue;                // block-uniform
        const int j = tid + t * 1024;
        int total;
        const int o = running + block_rank(keep[t], s_red, total);
        if (keep[t] && o < p.Rcap) {
            kept_index[(long)b * p.Rcap + o] = j;
            src_row[(long)b * rows_cap + o] = j;
            if (out_protect) out_protect[(long)b * rows_cap + o] = key[t] ? 1 : 0;
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
    u32x4* __restrict__ hidden_out, u32x4* __restrict__ k_out, u32x4* __restrict__ v_out, int text_done)
{
    const int o = blockIdx.x, b = blockIdx.y;
    const int rows_cap = p.Rcap + p.N;
    const int src = src_row[(long)b * rows_cap + o];
    if (src < 0 || (text_done && src >= p.Mv)) return;     // text rows may have been copied by the selection launch
    const int hv = p.C / 8, kv = p.H * p.d / 8;          // 16-byte vectors per row
    const u32x4* hs = hidden + ((long)b * p.L + src) * hv;
    const u32x4* ks = k + ((long)b * p.L + src) * kv;
    const u32x4* vs = v + ((long)b * p.L + src) * kv;
    u32x4* hd = hidden_out + ((long)b * rows_cap + o) * hv;
    u32x4* kd = k_out + ((long)b * rows_cap + o) * kv;
    u32x4* vd = v_out + ((long)b * rows_cap + o) * kv;
    // every source row is read once (streaming loads; the copies are read again by the next stage),
    // four vectors in flight
    auto copy2 = [&](const u32x4* __restrict__ s0, u32x4* __restrict__ d0, const u32x4* __restrict__ s1,
                     u32x4* __restrict__ d1, int n) {
        const int step = 2 * blockDim.x;
        for (int c = threadIdx.x; c < n; c += step) {
            const int c2 = c + blockDim.x;
            const bool two = c2 < n;
            const u32x4 a0 = __builtin_nontemporal_load(s0 + c), a1 = __builtin_nontemporal_load(s1 + c);
            u32x4 b0 = a0, b1 = a1;
            if (two) { b0 = __builtin_nontemporal_load(s0 + c2); b1 = __builtin_nontemporal_load(s1 + c2); }
            d0[c] = a0;
            d1[c] = a1;
            if (two) { d0[c2] = b0; d1[c2] = b1; }
        }
    };
    copy2(ks, kd, vs, vd, kv);
    const int half = (hv + 1) / 2;                   // the hidden row as two halves
    copy2(hs, hd, hs + half, hd + half, hv - half);
    if (hv & 1) {                                    // odd vector count: the first half has one more
        const int c = half - 1;
        if (threadIdx.x == 0) hd[c] = hs[c];
    }
}

// The same for K / V in other layouts: a row is gathered head slice by head slice (d contiguous
// elements each) from the input layout and scattered to the output layout.
__global__ __launch_bounds__(256) void prefill_compact_strided_kernel(
    PrefillDims p, const int32_t* __restrict__ src_row,
    const u32x4* __restrict__ hidden, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    u32x4* __restrict__ hidden_out, uint16_t* __restrict__ k_out, uint16_t* __restrict__ v_out, KvLayout out)
{
    const int o = blockIdx.x, b = blockIdx.y;
    const int rows_cap = p.Rcap + p.N;
    const int src = src_row[(long)b * rows_cap + o];
    if (src < 0) return;
    const int lph = p.d / 8;                             // 16-byte vectors per head slice
    const int kvn = p.H * lph;
    const long sbase = (long)b * p.kv.batch + (long)src * p.kv.token;
    const long dbase = (long)b * out.batch + (long)o * out.token;
    for (int c = threadIdx.x; c < kvn; c += blockDim.x) {
        const int h = c / lph, w = c - h * lph;
        const long so = sbase + (long)h * p.kv.head + w * 8, d_o = dbase + (long)h * out.head + w * 8;
        const u32x4 a = *reinterpret_cast<const u32x4*>(k + so);
        const u32x4 c2 = *reinterpret_cast<const u32x4*>(v + so);
        *reinterpret_cast<u32x4*>(k_out + d_o) = a;
        *reinterpret_cast<u32x4*>(v_out + d_o) = c2;
    }
    const int hv = p.C / 8;
    const u32x4* hs = hidden + ((long)b * p.L + src) * hv;
    u32x4* hd = hidden_out + ((long)b * rows_cap + o) * hv;
    for (int c = threadIdx.x; c < hv; c += blockDim.x) hd[c] = hs[c];
}

// Prompts of more than 128 text rows: V = sum, I = max over the launches' partial results (group 0 holds the result).
__global__ __launch_bounds__(256) void prefill_merge_groups_kernel(long n, int groups, float* __restrict__ V, float* __restrict__ I)
{
    const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    float v = V[e], m = I[e];
    for (int g = 1; g < groups; ++g) { v += V[g * n + e]; m = fmaxf(m, I[g * n + e]); }
    V[e] = v;
    I[e] = m;
}

struct PrefillWorkspace {
    float2* partial; float* cstat; bf16x8* qfrag; float* V; float* I; float* score; int32_t* src_row;
    size_t bytes;
};

#ifndef MD_RS_BLOCKS
#define MD_RS_BLOCKS 512   // target number of blocks of the row-statistics sweep
#endif
#ifndef MD_PF_NW
#define MD_PF_NW 4      // waves per block in the column-score sweep (measured: 4 beats 8 and 16)
#endif

int pick_chunks(int B, int H, int L, int ntg) {
    // enough (sample, head, chunk) blocks to cover the 256 CUs several times; chunks of whole tiles
    // about two resident blocks per CU (512 in all); at least 4 tiles per chunk so every wave has work
    const int tiles = (L + 31) / 32;
    int nch = (MD_RS_BLOCKS + B * H * ntg - 1) / (B * H * ntg);   // ntg: text groups, also spread over blocks
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
    w.cstat = c.take<float>((size_t)B * H * Npad);
    w.qfrag = c.take<bf16x8>((size_t)B * H * Npad * 16);      // [B][H][NB][KS][64] fragments, d <= 128
    const int groups = (Npad / 32 + 3) / 4;                    // column-score launches (128 text rows each)
    w.V = c.take<float>((size_t)groups * B * Mv);
    w.I = c.take<float>((size_t)groups * B * Mv);
    w.score = c.take<float>((size_t)B * Mv);
    w.src_row = c.take<int32_t>((size_t)B * (Rcap + N));
    w.bytes = c.off;
    return w;
}

template <int KS>
int launch_scores(const PrefillDims& p, const PrefillWorkspace& w, hipStream_t st, const void* q_txt, const void* k,
                  const uint8_t* vis_valid, const int32_t* txt_len, float scale_log2e) {
    constexpr int NW = MD_PF_NW;
    const int nbt = p.Npad / 32;                     // 32-row text blocks in all
    // sweep 1: a block covers two text blocks (one if there is only one)
    const int ntg = nbt == 1 ? 1 : (nbt + 1) / 2;
    dim3 g1(p.nch * ntg, p.H, p.B);
    if (nbt == 1)
        MD_LAUNCH("prefill_rowstats", st, (prefill_rowstats_kernel<1, KS>), g1, 256, 0,
            static_cast<const uint16_t*>(q_txt), static_cast<const uint16_t*>(k), vis_valid, txt_len, p, scale_log2e,
            w.partial, w.cstat, w.qfrag);
    else
        MD_LAUNCH("prefill_rowstats", st, (prefill_rowstats_kernel<2, KS>), g1, 256, 0,
            static_cast<const uint16_t*>(q_txt), static_cast<const uint16_t*>(k), vis_valid, txt_len, p, scale_log2e,
            w.partial, w.cstat, w.qfrag);
    if (p.nch > 1) {
        const long n = (long)p.B * p.H * p.Npad;
        MD_LAUNCH("prefill_cstat", st, (prefill_cstat_kernel), (unsigned)((n + 255) / 256), 256, 0,
            w.partial, txt_len, p, w.cstat);
    }
    // sweep 2: one launch per 128 text rows
    const int nt = (p.Mv + 31) / 32;
    dim3 g2(p.B % 8 == 0 || 8 % p.B != 0 ? nt * p.B : 8 * ((nt + 8 / p.B - 1) / (8 / p.B)));
    const long nv = (long)p.B * p.Mv;
    const int groups = (nbt + 3) / 4;
    for (int g = 0; g < groups; ++g) {
        const int nb0 = 4 * g, nbg = nbt - nb0 < 4 ? nbt - nb0 : 4;
        float* Vg = w.V + g * nv;
        float* Ig = w.I + g * nv;
#define MD_COLSCORE(NB_)                                                                                       \
        MD_LAUNCH("prefill_colscore", st, (prefill_colscore_kernel<NB_, KS, NW>), g2, 64 * NW, 0,                  \
            w.qfrag, static_cast<const uint16_t*>(k), vis_valid, txt_len, w.cstat, p, scale_log2e, nb0, Vg, Ig)
        if (nbg == 1) MD_COLSCORE(1);
        else if (nbg == 2) MD_COLSCORE(2);
        else if (nbg == 3) MD_COLSCORE(3);
        else MD_COLSCORE(4);
#undef MD_COLSCORE
    }
    if (groups > 1)
        MD_LAUNCH("prefill_merge_groups", st, (prefill_merge_groups_kernel), (unsigned)((nv + 255) / 256), 256, 0,
            nv, groups, w.V, w.I);
    return MD_OK;
}

}  // namespace
}  // namespace md

using namespace md;

extern "C" size_t mustdrop_prefill_filter_workspace_bytes(int B, int Mv, int N, int H, int Rcap) {
    if (B <= 0 || Mv <= 0 || N <= 0 || H <= 0 || Rcap <= 0) return 0;
    return carve_prefill(nullptr, B, Mv, N, H, Rcap).bytes;
}

namespace md {
namespace {

int prefill_filter_impl(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    const md_kv_layout* q_layout, const md_kv_layout* kv_layout, const md_kv_layout* kv_out_layout,
    void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    if (mode != MD_FILTER_BUDGET && mode != MD_FILTER_THRESHOLD) return fail(MD_EDTYPE, "prefill_filter: unknown mode %d", (int)mode);
    if (B <= 0 || Mv <= 0 || N <= 0 || H <= 0 || d <= 0 || C <= 0 || Rcap <= 0)
        return fail(MD_EINVAL, "prefill_filter: B, Mv, N, H, d, C, Rcap must be positive");
    if (!q_txt || !k || !v || !hidden || !hidden_out || !k_out || !v_out || !kept_index || !kept_count)
        return fail(MD_EINVAL, "prefill_filter: q_txt, k, v, hidden, the *_out tensors, kept_index and kept_count are required");
    if (d != 64 && d != 128) return fail(MD_ESHAPE, "prefill_filter: head dim %d not supported (64 or 128)", d);
    if (N > 1024) return fail(MD_ESHAPE, "prefill_filter: N=%d text tokens exceeds the limit of 1024", N);
    if (H > 128) return fail(MD_ESHAPE, "prefill_filter: H=%d heads exceeds the limit of 128", H);
    if ((long)B * (Mv + N) > (1l << 28)) return fail(MD_ESHAPE, "prefill_filter: too many tokens");
    if (C % 8) return fail(MD_EALIGN, "prefill_filter: a hidden row of C=%d bf16 is not a multiple of 16 bytes", C);
    if (std::isnan(softmax_scale) || std::isnan(gamma) || std::isnan(alpha)) return fail(MD_EINVAL, "prefill_filter: NaN parameter");
    if (!(softmax_scale > 0.f) || std::isinf(softmax_scale)) return fail(MD_EINVAL, "prefill_filter: softmax_scale must be positive and finite");
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
    KvLayout lq, lkv, lout;
    int lrc = read_layout("prefill_filter", "q_txt", q_layout, B, N, H, d, &lq);
    if (lrc == MD_OK) lrc = read_layout("prefill_filter", "k / v", kv_layout, B, (long)L, H, d, &lkv);
    if (lrc == MD_OK) lrc = read_layout("prefill_filter", "k_out / v_out", kv_out_layout, B, (long)Rcap + N, H, d, &lout);
    if (lrc != MD_OK) return lrc;
    if (lq.token > (1l << 26) || lkv.token > (1l << 26))
        return fail(MD_ESHAPE, "prefill_filter: token stride above 2^26 elements");
    const size_t kv_in = layout_extent_bytes(lkv, B, (long)L, H, d), h_in = (size_t)B * L * C * 2;
    const size_t kv_out = layout_extent_bytes(lout, B, (long)Rcap + N, H, d), h_out = (size_t)B * (Rcap + N) * C * 2;
    const void* ins[] = {k, v, hidden, q_txt};
    const size_t in_sz[] = {kv_in, kv_in, h_in, layout_extent_bytes(lq, B, N, H, d)};
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
    p.q = lq; p.kv = lkv;
    p.Npad = (N + 31) / 32 * 32;
    p.nch = pick_chunks(B, H, p.L, (p.Npad / 32 + 1) / 2);
    const int tiles = (p.L + 31) / 32;
    p.chunk = (tiles + p.nch - 1) / p.nch * 32;
    p.nch = (p.L + p.chunk - 1) / p.chunk;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float sl2 = softmax_scale * kLog2e;

    int rc = d == 128 ? launch_scores<8>(p, w, st, q_txt, k, vis_valid, txt_len, sl2)
                      : launch_scores<4>(p, w, st, q_txt, k, vis_valid, txt_len, sl2);
    if (rc != MD_OK) return rc;
    int32_t* src_row = out_ids ? out_ids : w.src_row;     // the row map doubles as the optional out_ids
    const bool dense_io = is_dense(lkv, (long)L, H, d) && is_dense(lout, (long)Rcap + N, H, d);
    TextRows tr{static_cast<const u32x4*>(hidden), static_cast<const u32x4*>(k), static_cast<const u32x4*>(v),
                static_cast<u32x4*>(hidden_out), static_cast<u32x4*>(k_out), static_cast<u32x4*>(v_out), 0};
    tr.enabled = (mode == MD_FILTER_BUDGET && dense_io && Mv <= 8192) ? 1 : 0;
    const int sel_blocks = B + (tr.enabled ? B * ((N + kTextRowsPerBlock - 1) / kTextRowsPerBlock) : 0);
#define MD_PSELECT_FAST(IPT_)                                                                               \
    MD_LAUNCH("prefill_select", st, (prefill_select_fast_kernel<IPT_>), sel_blocks, 1024, 0,        \
        p, w.V, w.I, vis_valid, txt_len, is_key, (int)mode, budget, gamma, alpha,                          \
        src_row, kept_index, kept_count, out_len, out_protect, score_global, score_indiv, tr)
    if (Mv <= 1024) MD_PSELECT_FAST(1);
    else if (Mv <= 2048) MD_PSELECT_FAST(2);
    else if (Mv <= 4096) MD_PSELECT_FAST(4);
    else if (Mv <= 8192) MD_PSELECT_FAST(8);
    else
        MD_LAUNCH("prefill_select", st, (prefill_select_kernel), B, 1024, 0,
            p, w.V, w.I, vis_valid, txt_len, is_key, (int)mode, budget, gamma, alpha,
            w.score, src_row, kept_index, kept_count, out_len, out_protect, score_global, score_indiv);
#undef MD_PSELECT_FAST
    dim3 gc(tr.enabled ? Rcap : Rcap + N, B);         // the text rows beyond the kept vision rows are already in place
    if (dense_io)
        MD_LAUNCH("prefill_compact", st, (prefill_compact_kernel), gc, 256, 0, p, src_row,
            static_cast<const u32x4*>(hidden), static_cast<const u32x4*>(k), static_cast<const u32x4*>(v),
            static_cast<u32x4*>(hidden_out), static_cast<u32x4*>(k_out), static_cast<u32x4*>(v_out), tr.enabled);
    else
        MD_LAUNCH("prefill_compact", st, (prefill_compact_strided_kernel), gc, 256, 0, p, src_row,
            static_cast<const u32x4*>(hidden), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
            static_cast<u32x4*>(hidden_out), static_cast<uint16_t*>(k_out), static_cast<uint16_t*>(v_out), lout);
    return check_launch("prefill_filter");
}

}  // namespace
}  // namespace md

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
    return prefill_filter_impl(q_txt, k, v, hidden, vis_valid, txt_len, is_key, B, Mv, N, H, d, C, softmax_scale, mode,
                               budget, gamma, alpha, Rcap, hidden_out, k_out, v_out, kept_index, kept_count, out_len,
                               out_protect, out_ids, score_global, score_indiv, nullptr, nullptr, nullptr,
                               workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_prefill_filter_strided(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    const md_kv_layout* q_layout, const md_kv_layout* kv_layout, const md_kv_layout* kv_out_layout,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return prefill_filter_impl(q_txt, k, v, hidden, vis_valid, txt_len, is_key, B, Mv, N, H, d, C, softmax_scale, mode,
                               budget, gamma, alpha, Rcap, hidden_out, k_out, v_out, kept_index, kept_count, out_len,
                               out_protect, out_ids, score_global, score_indiv, q_layout, kv_layout, kv_out_layout,
                               workspace, workspace_bytes, stream);
}
