// Stage 2 -- prefill (Sec. 3.4): text-to-vision attention scores, the dual filter (Eq. 8-10) and
// token drop (stable compaction of hidden states, K and V).
//
// The column statistics V_j = sum_i a_ij and I_j = max_i a_ij need the row softmax normaliser of
// every text row over the WHOLE key axis, and the head mean has to be taken before the max over
// text rows.  The normalisers are a by-product of the layer's own attention (Sec. 3.4): a caller
// that has them (row_lse) pays one sweep over K; otherwise a first sweep computes them:
//   prefill_rowstats_kernel  per (sample, head, key chunk): S = K Q^T on the MFMA units, online
//                            (max, sum-exp) per text row -> row statistics (prefill_cstat_kernel
//                            merges the chunks); with row_lse only prefill_qpack_kernel runs
//   prefill_colscore_kernel  persistent blocks over units of (64 or 128 vision keys, one head): recompute
//                            S, p = exp(s - m)/Z, accumulate the head mean a[i][j] of such a key tile
//                            in registers; a block's share of a tile is written as one piece
//   prefill_colfix_kernel    sums a tile's pieces in a fixed order, column sum / max -> V_j, I_j
// The N x Mv probability matrix of a head is never written to memory.
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
constexpr int kMaxChunks = 8;                        // key chunks per (sample, head) in the row-statistics sweep, at most

struct PrefillDims {
    int B, Mv, N, H, d, C, L;
    int nch;          // key chunks per (sample, head) in the row-statistics sweep
    int chunk;        // keys per chunk (multiple of 128)
    int Npad;         // 32 * (number of 32-row text blocks)
    int Rcap;
    KvLayout q, kv;   // element strides of q_txt and of k (v shares them)
};

// key row of accumulator register r in the 32x32 result tile
__device__ __forceinline__ int tile_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

#define MD_VM_WAIT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Every LDS access of this wave has completed, then the block barrier.  (The loads that write LDS
// directly are counted by vmcnt: the caller waits for those itself.)
__device__ __forceinline__ void block_sync_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Rows of an MFMA operand (one head slice of a key or a text query: 16*KS bf16 = CH chunks of 16
// bytes) on their way from global memory to MFMA fragments, through LDS.
//   global -> LDS  buffer loads that write LDS directly (no staging registers): a wave instruction
//                  moves 1 KiB = RPL whole rows, coalesced; rows outside the buffer resource's range
//                  are never fetched.
//   LDS layout     rows unpadded (pitch ROWB); the chunk a lane fetches for position `pos` of row
//                  `row` is pos ^ swz(row), so that the 128-bit fragment reads below (32 rows, one
//                  chunk index) spread over all banks.
//   LDS -> frags   lane (g = lane/32, r = lane%32) of the 32x32x16 MFMA holds row r, chunks 2*ks+g.
template <int KS>
struct LdsRows {
    static constexpr int CH = 2 * KS;
    static constexpr int ROWB = CH * 16;             // 256 (d = 128) or 128 (d = 64) bytes
    static constexpr int RPL = kWave / CH;           // rows per load instruction
    static_assert(KS == 4 || KS == 8, "rows of 128 or 256 bytes");
    __device__ static __forceinline__ int swz(int row) { return KS == 8 ? (row & 15) : ((row >> 1) & 7); }

    // One wave instruction: rows slot_row .. slot_row+RPL-1 of the LDS block at `lds_base` (wave-uniform)
    // receive the global rows grow0+slot_row.. of the matrix behind `rs` (rows row_bytes apart).
    // `live` (wave-uniform) false: nothing is fetched.
    __device__ static __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, uint32_t row_bytes, int grow0, int slot_row,
                                                 char* lds_base, int lane, bool live) {
        const int row = slot_row + lane / CH, pos = lane % CH;
        const uint32_t off = live ? (uint32_t)(grow0 + row) * row_bytes + (uint32_t)((pos ^ swz(row)) << 4) : 0xFFFFFF00u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(lds_base + slot_row * ROWB), 16, off, 0, 0, 0);
    }
    // LDS byte address of this lane's fragment row in the 32-row tile at `tile` (aligned to 32*ROWB),
    // with the swizzle and the lane half folded in; chunk index ks is applied with XOR.
    __device__ static __forceinline__ uint32_t frag_base(const char* tile, int lane) {
        const int r = lane & 31, g = lane >> 5;
        const uint32_t a = (uint32_t)(uintptr_t)(lds_ptr_t)const_cast<char*>(tile);
        return (a + r * ROWB) ^ (uint32_t)((g << 4) ^ (swz(r) << 4));
    }
    // the KS fragments of a tile; returns once they are in registers
    __device__ static __forceinline__ void frags(uint32_t fb, bf16x8 (&f)[KS]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint32_t a;
            asm volatile("v_xor_b32 %1, %2, %3\n\tds_read_b128 %0, %1" : "=v"(f[ks]), "=&v"(a) : "v"(ks << 5), "v"(fb) : "memory");
        }
        if constexpr (KS == 8)
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]) :: "memory");
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) :: "memory");
    }
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_buffer(const uint16_t* base, long rows, long row_stride, int d) {
    // rows [0, rows) of `d` elements each, row_stride elements apart; anything beyond reads as "not there"
    const long bytes = rows > 0 ? ((rows - 1) * row_stride + d) * 2 : 0;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, (int)bytes, 0x00020000);
}

// Vision rows that matter.  Vision tokens arrive with a validity mask; after the vision-encoder stage
// merged tokens away the valid ones of a sample are a prefix and the rest of its Mv slots is padding.
// Both sweeps skip the slots behind the last valid one: eff = min(Mv, round_up32(last valid + 1))
// (0 when no slot is valid).  Any other pattern of invalid slots is still handled key by key.
// Per-thread part: the largest index this thread saw set among [0, n), or -1.
__device__ __forceinline__ int last_set_partial(const uint8_t* v, int n, int tid, int nthreads) {
    int last = -1;
    const int head = min(n, (int)((16 - ((uintptr_t)v & 15)) & 15));     // bytes before 16-byte alignment
    if (tid < head && v[tid]) last = tid;
    const int nvec = (n - head) / 16;
    const uint4* pv = reinterpret_cast<const uint4*>(v + head);
    for (int q = tid; q < nvec; q += nthreads) {
        const uint4 w = pv[q];
        const int base = head + q * 16;
        if (w.x) last = base + ((31 - __clz((int)w.x)) >> 3);
        if (w.y) last = base + 4 + ((31 - __clz((int)w.y)) >> 3);
        if (w.z) last = base + 8 + ((31 - __clz((int)w.z)) >> 3);
        if (w.w) last = base + 12 + ((31 - __clz((int)w.w)) >> 3);
    }
    for (int j = head + nvec * 16 + tid; j < n; j += nthreads)
        if (v[j]) last = j;
    return last;
}
__device__ __forceinline__ int wave_max_int(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ int effective_rows(int last, int Mv) { return last < 0 ? 0 : min(Mv, (last + 32) & ~31); }

// Row statistics folded into one constant: a probability of the head mean is
// exp2(s*scale*log2e + c) with c = -m - log2(Z) - log2(H); text rows beyond txt_len get -inf (-> 0).
__device__ __forceinline__ float fold_stats(float m, float z, bool row_ok, int H) {
    return (row_ok && z > 0.f) ? -m - fast_log2(z) - fast_log2((float)H) : -INFINITY;
}

// The 32 text-query rows i0.. of head slice `qb` as MFMA fragments: global -> this wave's LDS tile ->
// registers.  Rows at or beyond `tl` come out as zero rows.
template <int KS>
__device__ __forceinline__ void issue_query_rows(const uint16_t* qb, long tok_stride, int d, int i0, int tl, char* tile, int lane) {
    using T = LdsRows<KS>;
    const __amdgpu_buffer_rsrc_t rq = row_buffer(qb, tl, tok_stride, d);
#pragma unroll
    for (int t = 0; t < 32 / T::RPL; ++t) T::issue(rq, (uint32_t)(tok_stride * 2), i0, t * T::RPL, tile, lane, true);
}
template <int KS>
__device__ __forceinline__ void read_query_frags(int i0, int tl, const char* tile, int lane, bf16x8 (&qf)[KS]) {
    using T = LdsRows<KS>;
    MD_VM_WAIT(0);
    T::frags(T::frag_base(tile, lane), qf);
    const bool row_ok = i0 + (lane & 31) < tl;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        if (!row_ok) qf[ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
}
template <int KS>
__device__ __forceinline__ void load_query_frags(const uint16_t* qb, long tok_stride, int d, int i0, int tl, char* tile,
                                                 int lane, bf16x8 (&qf)[KS]) {
    issue_query_rows<KS>(qb, tok_stride, d, i0, tl, tile, lane);
    read_query_frags<KS>(i0, tl, tile, lane, qf);
}

// ---------------------------------------------------------------------------------------------
// Sweep 1: row statistics.  Block = (key chunk x text group, head, sample), 4 waves.  The waves of a
// block share every K tile through LDS: wave w works on text block w % NBW of the group and on key
// tile w / NBW of the TW = 4/NBW tiles in flight per step, so a wave keeps the fragments of ONE
// 32-row text block in registers and K is read once per block.  K tiles stream through S LDS slots
// (filled S-1 steps ahead, no staging registers); one block barrier per step.  Inside a step the
// MFMA chain of the current tile is issued before the softmax arithmetic of the previous one (two
// accumulators), so the matrix unit and the vector ALUs overlap within a wave.
// Chunk 0 also stores the text-query fragments in fragment-major order (qfrag), rows beyond txt_len
// zeroed, for the second sweep.
template <int KS>
__device__ __forceinline__ f32x16 score_tile(const bf16x8 (&kf)[KS], const bf16x8 (&qf)[KS]) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], acc, 0, 0, 0);
    return acc;
}

// Online (max, sum of exp2) update of one lane's text row with the 16 keys it holds of a tile.
// Fast form: every key of the tile is visible -- straight-line code (so that the compiler can
// interleave it with the MFMA chain of the next tile), maximum and sum as trees.
__device__ __forceinline__ void online_update_all(const f32x16& acc, float scale_log2e, float& m, float& z) {
    const float b0 = fmaxf(fmaxf(acc[0], acc[1]), acc[2]), b1 = fmaxf(fmaxf(acc[3], acc[4]), acc[5]);
    const float b2 = fmaxf(fmaxf(acc[6], acc[7]), acc[8]), b3 = fmaxf(fmaxf(acc[9], acc[10]), acc[11]);
    const float b4 = fmaxf(fmaxf(acc[12], acc[13]), acc[14]);
    const float bm = fmaxf(fmaxf(fmaxf(b0, b1), b2), fmaxf(fmaxf(b3, b4), acc[15]));
    const float mn = fmaxf(m, bm * scale_log2e);     // the scale is positive: applied after the maximum
    const float nmn = -mn;
    float e[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] = fast_exp2(fmaf(acc[r], scale_log2e, nmn));
    const float s = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7])) +
                    (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
    z = fmaf(z, fast_exp2(m - mn), s);               // m = -inf at the first tile: exp2(-inf) = 0
    m = mn;
}
// General form: `vis` bit r set = accumulator r is a visible key.
__device__ __forceinline__ void online_update_masked(f32x16 acc, uint32_t vis, float scale_log2e, float& m, float& z) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (!((vis >> r) & 1u)) acc[r] = -INFINITY;
    float bm = acc[0];
#pragma unroll
    for (int r = 1; r < 16; r += 2) bm = fmaxf(fmaxf(bm, acc[r]), acc[r + 1 < 16 ? r + 1 : r]);
    const float mn = fmaxf(m, bm * scale_log2e);
    if (mn > -INFINITY) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            s0 += fast_exp2(fmaf(acc[r], scale_log2e, -mn));
            s1 += fast_exp2(fmaf(acc[r + 1], scale_log2e, -mn));
        }
        z = fmaf(z, fast_exp2(m - mn), s0 + s1);
        m = mn;
    }
}

// The compiler's scheduler is asked to issue one MFMA, then a few vector and transcendental
// instructions, and so on: a wave issues in order, and a chain of dependent MFMAs issued back to back
// would hold up the independent vector work behind it.
template <int KS>
__device__ __forceinline__ void interleave_mfma_valu() {
#pragma unroll
    for (int q = 0; q < KS; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 48 / KS, 0);
        __builtin_amdgcn_sched_group_barrier(0x400, 16 / KS, 0);
    }
}

template <int NBW, int TW, int KS>
__global__ __launch_bounds__(64 * NBW * TW) void prefill_rowstats_kernel(
    const uint16_t* __restrict__ q_txt, const uint16_t* __restrict__ k,
    const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len, PrefillDims p, float scale_log2e,
    float2* __restrict__ partial, float* __restrict__ cstat, bf16x8* __restrict__ qfrag, int32_t* __restrict__ mv_eff)
{
    using T = LdsRows<KS>;
    // NBW wave columns (one 32-row text block each) x TW tile lanes (one 32-key tile of a step each): four waves,
    // or eight (NBW = 4, TW = 2) where one block then covers what two chunk blocks would and their statistics meet
    // in LDS instead of in a separate kernel
    constexpr int NW = NBW * TW;
    // LDS slots.  The eight-wave form runs with two (one step in flight while one is worked on): with more
    // requests outstanding per CU the sweep gets slower, not faster, when K comes from HBM (46.3 against 47.9 us)
    constexpr int S = TW == 1 ? 4 : (NW == 8 ? 2 : 3);
    constexpr int SLOT_ROWS = 32 * TW, SLOT_BYTES = SLOT_ROWS * T::ROWB;
    constexpr int NLW = SLOT_ROWS / T::RPL / NW;      // load instructions per wave and step
    constexpr int QBYTES = NBW * 32 * T::ROWB;        // the block's query tiles during the prologue (one per wave column)
    __shared__ __attribute__((aligned(1024))) char s_k[S * SLOT_BYTES];
    __shared__ __attribute__((aligned(1024))) char s_q[QBYTES];
    __shared__ float s_m[NW][32], s_z[NW][32];
    __shared__ int s_last[NW];
    const int lane = lane_id(), wv = wave_id();
    const int nbw = wv % NBW, tw = wv / NBW;
    const int ch = blockIdx.x % p.nch, tg = blockIdx.x / p.nch, h = blockIdx.y, b = blockIdx.z;
    const int nbg = tg * NBW + nbw;                   // 32-row text block of this wave
    const int i0 = 32 * nbg;
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    const uint16_t* kb = k + (long)b * p.kv.batch + (long)h * p.kv.head;
    const uint16_t* qb = q_txt + (long)b * p.q.batch + (long)h * p.q.head;
    const uint8_t* vb = vis_valid ? vis_valid + (long)b * p.Mv : nullptr;
    const __amdgpu_buffer_rsrc_t rk = row_buffer(kb, p.L, p.kv.token, p.d);
    const uint32_t krow = (uint32_t)(p.kv.token * 2);

    // The sweep runs over "effective" key positions e: the Me vision rows that matter (see
    // effective_rows), then the N text rows; e >= Me is row e + jump of K.  Me is a multiple of 32 (or
    // Mv itself), so a 32-key tile never straddles the jump.  The nch blocks of a (sample, head) take the
    // SLOT_ROWS-key steps in turn (block ch: steps ch, ch + nch, ...): their shares are even whatever Me is,
    // and a block knows where its first steps lie before Me has been found.
    int Me = p.Mv, jump = 0, c1 = 0, nit = 0;
    auto plan = [&]() {
        jump = p.Mv - Me;
        c1 = Me + p.N;
        const int steps = (c1 + SLOT_ROWS - 1) / SLOT_ROWS;
        nit = steps > ch ? (steps - ch + p.nch - 1) / p.nch : 0;          // steps of this block
    };
    auto step_row0 = [&](int g) { return (ch + g * p.nch) * SLOT_ROWS; };  // effective position of step g's first key
    // step g's tiles go to slot g % S
    auto issue_step = [&](int g) {
        char* slot = s_k + (g % S) * SLOT_BYTES;
        const int row0 = step_row0(g);
#pragma unroll
        for (int t = 0; t < NLW; ++t) {
            const int sr = (t * NW + wv) * T::RPL;
            T::issue(rk, krow, row0 + (row0 + sr >= Me ? jump : 0), sr, slot, lane, true);
        }
    };
    // Validity of the 32 keys of this wave's tile in the steps g0 .. g0+63: lane l fetches the 32 mask bytes of
    // step g0 + l and turns them into one word (bit r = key r of the tile is a valid vision token; bytes beyond
    // the sample's Mv slots count as invalid), so a step gets its mask with one lane read and the whole batch
    // costs one round trip.  (A load inside the steady loop would have the compiler wait for everything in
    // flight, the K tiles included, once per step.)
    auto key_valid_masks = [&](int g0) -> uint32_t {
        if (!vb) return 0xFFFFFFFFu;
        const long e0 = (long)step_row0(g0 + lane) + tw * 32;         // first key of the tile; a multiple of 32
        uint32_t mask = 0;
        if ((reinterpret_cast<uintptr_t>(vb) & 3) == 0) {             // block-uniform: the mask row is word-aligned
            const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(vb), 0, (p.Mv + 3) & ~3, 0x00020000);
            uint32_t w[8];
            const int off = (int)min(e0, (long)((p.Mv + 3) & ~3));    // beyond the row: out of the buffer's range, reads 0
#pragma unroll
            for (int q = 0; q < 8; ++q) w[q] = __builtin_amdgcn_raw_buffer_load_b32(rv, off + 4 * q, 0, 0);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                mask |= (((w[q] & 0xFFu) ? 1u : 0u) | ((w[q] & 0xFF00u) ? 2u : 0u) | ((w[q] & 0xFF0000u) ? 4u : 0u) |
                         ((w[q] & 0xFF000000u) ? 8u : 0u)) << (4 * q);
        } else {
            for (int r = 0; r < 32; ++r) mask |= (vb[min(e0 + r, (long)p.Mv - 1)] != 0 ? 1u : 0u) << r;
        }
        const long left = (long)p.Mv - e0;                            // slots of the row from this tile on
        if (left < 32) mask &= left <= 0 ? 0u : (1u << left) - 1u;
        return mask;
    };

    // Prologue, one round trip: the query tiles (each wave column's tile, its rows split among the column's
    // waves), the scan of the validity mask, and the first S-1 steps of K all go out together.  With a mask the
    // rows that matter (Me) are not known yet: the steps are requested as if they lay below Me, which holds
    // unless the sample has fewer than (S-1) * nch * SLOT_ROWS rows that matter; then they are requested again.
    plan();
#pragma unroll
    for (int g = 0; g < S - 1; ++g)
        if (g < nit) issue_step(g);
    {
        const __amdgpu_buffer_rsrc_t rq = row_buffer(qb, tl, p.q.token, p.d);
#pragma unroll
        for (int t = tw; t < 32 / T::RPL; t += TW)    // this wave's share of its column's 32 query rows
            T::issue(rq, (uint32_t)(p.q.token * 2), i0, t * T::RPL, s_q + nbw * 32 * T::ROWB, lane, true);
    }
    if (vb) {
        const int last = wave_max_int(last_set_partial(vb, p.Mv, threadIdx.x, 64 * NW));
        if (lane == 0) s_last[wv] = last;
    }
    uint32_t vismasks = key_valid_masks(0);           // (its loads belong to the same round trip)
    MD_VM_WAIT(0);
    block_sync_lds();                                 // query tiles complete, mask scanned, first steps landed
    bf16x8 qf[KS];
    read_query_frags<KS>(i0, tl, s_q + nbw * 32 * T::ROWB, lane, qf);
    if (vb) {
        const int nit_guess = nit;
        int last = s_last[0];
#pragma unroll
        for (int w2 = 1; w2 < NW; ++w2) last = max(last, s_last[w2]);
        Me = effective_rows(last, p.Mv);
        plan();
        if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0) mv_eff[b] = Me;   // for the second sweep
        const int ahead = min(S - 1, max(nit, nit_guess));
        if (ahead > 0 && step_row0(ahead - 1) + SLOT_ROWS > Me) {            // a requested step reaches beyond Me: again, with the jump
#pragma unroll
            for (int g = 0; g < S - 1; ++g)
                if (g < nit) issue_step(g);
        }
    } else if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0) {
        mv_eff[b] = p.Mv;
    }

    float m = -INFINITY, z = 0.f;
    const int i = i0 + (lane & 31);
    // what the arithmetic of a finished tile needs besides its accumulator
    struct Pending { bool all; uint32_t vis; };
    auto visibility = [&](int g) -> Pending {
        const int j0 = step_row0(g) + tw * 32;        // effective position of the tile's first key
        // the tile's 32 keys (vision keys only): valid, and below the rows that matter
        uint32_t vmask = (uint32_t)__builtin_amdgcn_readlane((int)vismasks, g & 63);
        if (j0 + 32 > Me) vmask &= j0 >= Me ? 0u : (1u << (Me - j0)) - 1u;
        Pending pd;
        pd.all = j0 + 32 <= Me && vmask == 0xFFFFFFFFu;
        pd.vis = 0xFFFFu;
        if (!pd.all) {
            uint32_t bits = 0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile_row(r, lane), j = j0 + row;
                const bool vis = j < Me ? ((vmask >> row) & 1u) : (j < c1 && (j - Me) <= i);
                bits |= (vis ? 1u : 0u) << r;
            }
            pd.vis = bits;
        }
        return pd;
    };
    // Step g: wait for its tiles, refill the slot of step g-1, fragments of this wave's tile.
    auto fetch = [&](int g, bf16x8 (&kf)[KS]) {
        if (g + S - 2 < nit) { MD_VM_WAIT((S - 2) * NLW); } else { MD_VM_WAIT(0); }   // this wave's part of step g has landed
        block_sync_lds();                             // ... and everyone else's; step g-1's slot is free
        if (g + S - 1 < nit) issue_step(g + S - 1);
        T::frags(T::frag_base(s_k + (g % S) * SLOT_BYTES + tw * 32 * T::ROWB, lane), kf);
    };
    // The MFMA chain of step g is issued together with the arithmetic on the tile of step g-1.
    auto step = [&](int g, f32x16& acc_new, const f32x16& acc_old, Pending& pend) {
        bf16x8 kf[KS];
        fetch(g, kf);
        if (pend.all) {
            acc_new = score_tile<KS>(kf, qf);
            online_update_all(acc_old, scale_log2e, m, z);
            interleave_mfma_valu<KS>();
        } else {
            acc_new = score_tile<KS>(kf, qf);
            online_update_masked(acc_old, pend.vis, scale_log2e, m, z);
        }
        pend = visibility(g);
        if ((g & 63) == 63 && g + 1 < nit) vismasks = key_valid_masks(g + 1);   // (drains the loads in flight: once per 64 steps)
    };
    f32x16 accA, accB;
    Pending pend{true, 0xFFFFu};
    if (nit > 0) {
        bf16x8 kf[KS];
        fetch(0, kf);
        accA = score_tile<KS>(kf, qf);
        pend = visibility(0);
    }
    int g = 1;
    for (; g + 1 < nit; g += 2) {
        step(g, accB, accA, pend);
        step(g + 1, accA, accB, pend);
    }
    if (g < nit) {
        step(g, accB, accA, pend);
        if (pend.all) online_update_all(accB, scale_log2e, m, z); else online_update_masked(accB, pend.vis, scale_log2e, m, z);
    } else if (nit > 0) {
        if (pend.all) online_update_all(accA, scale_log2e, m, z); else online_update_masked(accA, pend.vis, scale_log2e, m, z);
    }
    MD_VM_WAIT(0);
    // the fragment-major copy of the text queries for the second sweep (here, where no load waits behind the stores)
    if (ch == 0 && tw == 0 && nbg < p.Npad / 32) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qfrag[((((long)b * p.H + h) * (p.Npad / 32) + nbg) * KS + ks) * kWave + lane] = qf[ks];
    }
    // merge the two lane halves (same text row, the other 16 keys), then the tile lanes
    {
        const float mo = __shfl_xor(m, 32, kWave), zo = __shfl_xor(z, 32, kWave);
        const float mn = fmaxf(m, mo);
        float zn = 0.f;
        if (mn > -INFINITY) zn = z * fast_exp2(m - mn) + zo * fast_exp2(mo - mn);
        if (lane < 32) { s_m[wv][lane] = mn; s_z[wv][lane] = zn; }
    }
    __syncthreads();
    if (threadIdx.x < 32 * NBW) {
        const int nb = threadIdx.x >> 5, r = threadIdx.x & 31;
        float mn = -INFINITY;
#pragma unroll
        for (int t = 0; t < TW; ++t) mn = fmaxf(mn, s_m[t * NBW + nb][r]);
        float zn = 0.f;
        if (mn > -INFINITY) {
#pragma unroll
            for (int t = 0; t < TW; ++t) zn += s_z[t * NBW + nb][r] * fast_exp2(s_m[t * NBW + nb][r] - mn);
        }
        const int ii = 32 * (tg * NBW + nb) + r;
        if (ii < p.Npad) {
            if (p.nch == 1)     // the only chunk: fold the statistics right away (see fold_stats)
                cstat[((long)b * p.H + h) * p.Npad + ii] = fold_stats(mn, zn, ii < tl, p.H);
            else
                partial[(((long)b * p.H + h) * p.nch + ch) * p.Npad + ii] = make_float2(mn, zn);
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

// The text-query fragments alone (the caller brought the row statistics, so sweep 1 does not run):
// one wave per (sample, head, 32-row text block).
template <int KS>
__global__ __launch_bounds__(256) void prefill_qpack_kernel(
    const uint16_t* __restrict__ q_txt, const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ txt_len,
    const float* __restrict__ row_lse, PrefillDims p, bf16x8* __restrict__ qfrag, float* __restrict__ cstat,
    int32_t* __restrict__ mv_eff)
{
    using T = LdsRows<KS>;
    __shared__ __attribute__((aligned(1024))) char s_q[4 * 32 * T::ROWB];
    __shared__ int s_last[4];
    const int lane = lane_id(), wv = wave_id();
    const int nbt = p.Npad / 32;
    const long items = (long)p.B * p.H * nbt;
    const long item_blocks = (items + 3) / 4;
    if ((long)blockIdx.x >= item_blocks) {            // the last B blocks: the vision rows that matter, per sample
        const int b = (int)(blockIdx.x - item_blocks);
        int last = p.Mv - 1;
        if (vis_valid) {
            last = wave_max_int(last_set_partial(vis_valid + (long)b * p.Mv, p.Mv, threadIdx.x, 256));
            if (lane == 0) s_last[wv] = last;
            __syncthreads();
            last = max(max(s_last[0], s_last[1]), max(s_last[2], s_last[3]));
        }
        if (threadIdx.x == 0) mv_eff[b] = effective_rows(last, p.Mv);
        return;
    }
    const long item = (long)blockIdx.x * 4 + wv;
    if (item >= items) return;
    const int nbg = (int)(item % nbt), h = (int)(item / nbt % p.H), b = (int)(item / nbt / p.H);
    const int tl = txt_len ? min(max(txt_len[b], 0), p.N) : p.N;
    bf16x8 qf[KS];
    load_query_frags<KS>(q_txt + (long)b * p.q.batch + (long)h * p.q.head, p.q.token, p.d, 32 * nbg, tl,
                         s_q + wv * 32 * T::ROWB, lane, qf);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qfrag[(item * KS + ks) * kWave + lane] = qf[ks];
    // the caller's log-sum-exp (natural log, over the keys the row sees) as the folded statistic:
    // exp(s*scale - lse) / H = exp2(s*scale*log2e + c), c = -lse*log2e - log2(H)
    if (lane < 32) {
        const int i = 32 * nbg + lane;
        const float lse = row_lse[((long)b * p.H + h) * p.N + min(i, p.N - 1)];
        cstat[((long)b * p.H + h) * p.Npad + i] = i < tl ? -lse * kLog2e - fast_log2((float)p.H) : -INFINITY;
    }
}

// ---------------------------------------------------------------------------------------------
// Sweep 2: head-mean probabilities.  The work is cut into units (kb vision keys of a sample, one head; kb = 64,
// or 128 with a single text block: smaller key groups mean smaller pieces and less to hand over, at the price of
// the query fragments being fetched from L2 more often per K byte; 64 measured best where a block holds two or
// four text blocks, 32 worse);
// a persistent grid of P blocks (one or two per CU) takes equal, contiguous runs of units
// [p*U/P, (p+1)*U/P), ordered (sample, key group, head), whatever the shape: no block count has to
// match the chip.  A block of 4 waves holds a [kb keys x 32*NBW text rows] tile of a[i][j] in
// registers (wave w: text block w % NBW, the KT key tiles of tile lane w / NBW) and adds one head's
// probabilities per unit.  Per unit the kb K rows go global -> registers -> LDS (two slots; the rows
// of unit u+2 are requested while unit u is worked on), the wave's text-query fragments come from
// qfrag (coalesced).  The row statistics are folded into one constant per (head, text row):
// p = exp2(s*scale*log2e + c), c = -m - log2(Z*H) (cstat: from sweep 1, or from the caller's
// log-sum-exp), so a probability costs one FMA and one exp2.  The MFMA chain of a key tile is issued together with the exp2 work of the tile before it.
// Where a run leaves a key group (or ends) the block writes its head-partial sums a[j][i] as one
// "piece" (fp32, key-major); prefill_colfix_kernel adds a key group's pieces in a fixed order and
// reduces over the text rows (Eq. 8 / Eq. 10).  Which block holds which piece is a function of the
// shapes alone, so the result does not depend on timing.
struct ColPlan { int P; long U; int nkg; int Gmax; int kb; };   // kb: vision keys per unit (a power of two)

__host__ __device__ __forceinline__ int unit_block(long u, int P, long U) { return (int)(((u + 1) * P - 1) / U); }

// The same decomposition over the key groups that matter (mv_eff, one entry per sample; written by the
// kernel before this sweep): sample b owns the tiles [tile0(b), tile0(b) + ceil(mv_eff[b] / 128)).
// Fewer units than the host planned for means fewer blocks at work only where a key group would
// otherwise be cut into more pieces than the workspace holds (Gmax).
struct ColRun { long U; int P; int tile0; int nk; };
__device__ __forceinline__ int key_groups(int rows, int kb) { return (rows + kb - 1) / kb; }
__device__ __forceinline__ ColRun effective_run(const int32_t* __restrict__ mv_eff, int B, int H, ColPlan cp, int bq) {
    int tiles = 0, tile0 = 0, nk = 0;
    for (int b = 0; b < B; ++b) {
        const int n = key_groups(mv_eff[b], cp.kb);
        if (b == bq) { tile0 = tiles; nk = n; }
        tiles += n;
    }
    ColRun r;
    r.U = (long)tiles * H;
    long P = (long)(cp.Gmax - 1) * tiles;             // pieces per key group <= ceil(H*P/U) + 1 <= Gmax
    if (cp.Gmax >= H || P > cp.P) P = cp.P;
    if (P >= 8) P &= ~7L;                             // whole rounds over the 8 XCDs
    if (P < 1) P = 1;
    r.P = (int)P;
    r.tile0 = tile0;
    r.nk = nk;
    return r;
}

template <int NBW, int KT, int KS>
__global__ __launch_bounds__(256, 2) void prefill_colscore_kernel(
    const bf16x8* __restrict__ qfrag, const uint16_t* __restrict__ k, const float* __restrict__ cstat,
    const int32_t* __restrict__ mv_eff, PrefillDims p, ColPlan cp, float scale_log2e, int tgrp, float* __restrict__ apart)
{
    constexpr int TW = 4 / NBW;
    constexpr int KB = 32 * TW * KT;                  // keys per unit (= cp.kb)
    constexpr int CH = 2 * KS;                        // 16-byte chunks per row
    constexpr int PITCH = CH * 16 + 16;               // padded row pitch: conflict-free 128-bit accesses
    constexpr int SLOT_BYTES = KB * PITCH;
    constexpr int RPL = kWave / CH;                   // rows per load instruction
    constexpr int NLW = KB / RPL / 4;                 // load instructions per wave and unit
    __shared__ __attribute__((aligned(16))) char s_k[2 * SLOT_BYTES];
    const int lane = lane_id(), wv = wave_id();
    const int nbw = wv % NBW, tw = wv / NBW;
    // Blocks go round-robin over the 8 XCDs (each with its own L2): the blocks of one XCD take neighbouring
    // runs, so a sample's query fragments are fetched into one or two L2s, not all eight.
    const ColRun run = effective_run(mv_eff, p.B, p.H, cp, -1);
    const int P = run.P;
    const long U = run.U;
    if ((int)blockIdx.x >= P) return;
    const int pb = (P % 8 == 0) ? (int)(blockIdx.x % 8) * (P / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    const long u0 = (long)pb * U / P, u1 = (long)(pb + 1) * U / P;
    if (u0 >= u1) return;
    const int nbt = p.Npad / 32;
    const int nbg = tgrp * NBW + nbw;                 // 32-row text block of this wave (may lie beyond the prompt)
    const bool has_rows = nbg < nbt;
    const int nbc = has_rows ? nbg : 0;
    const int i = 32 * nbc + (lane & 31);
    const long tok_stride = p.kv.token;

    // unit u = (tile, head); tile = (sample, key group), counted over the key groups that matter.  The
    // block walks its run with three cursors (the unit being worked on, the one whose fragments are
    // requested, the one whose K rows are requested), each advanced without divisions.
    struct Unit { int b, kg, h, nk, t; };             // nk: key groups of sample b; t: tile index
    auto unit_at = [&](long u) -> Unit {
        Unit x;
        x.t = (int)(u / p.H);
        x.h = (int)(u - (long)x.t * p.H);
        int first = 0;
        x.b = 0; x.kg = 0; x.nk = 1;
        for (int b = 0; b < p.B; ++b) {
            const int n = key_groups(mv_eff[b], KB);
            if (x.t >= first && x.t < first + n) { x.b = b; x.kg = x.t - first; x.nk = n; }
            first += n;
        }
        return x;
    };
    auto advance = [&](Unit& x) {
        if (++x.h == p.H) {
            x.h = 0;
            ++x.t;
            if (++x.kg == x.nk) {
                x.kg = 0;
                do { ++x.b; x.nk = x.b < p.B ? key_groups(mv_eff[x.b], KB) : 1; } while (x.nk == 0);
            }
        }
    };
    // This wave's share of a unit's K rows: NLW x 1 KiB; rows beyond the last vision key repeat it.
    // (`live` false, past the end of the run: every lane reads the same 16 bytes -- the loads stay
    // unconditional, so the compiler can count the loads in flight exactly.)
    auto load_k = [&](const Unit& x, bool live, u32x4 (&st)[NLW]) {
        const uint16_t* kb = k + (long)x.b * p.kv.batch + (long)x.h * p.kv.head + (live ? (lane % CH) * 8 : 0);
#pragma unroll
        for (int t = 0; t < NLW; ++t) {
            const int row = live ? min(x.kg * KB + (t * 4 + wv) * RPL + lane / CH, p.Mv - 1) : 0;
            // the last read of these rows (sweep 1 read them with plain loads, so part of them is still in the
            // Infinity Cache): streaming loads, which leave the cache to data that is used again
            st[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + (long)row * tok_stride));
        }
    };
    auto store_k = [&](int slot, const u32x4 (&st)[NLW]) {
        char* base = s_k + slot * SLOT_BYTES + (lane / CH) * PITCH + (lane % CH) * 16;
#pragma unroll
        for (int t = 0; t < NLW; ++t) *reinterpret_cast<u32x4*>(base + (t * 4 + wv) * RPL * PITCH) = st[t];
    };
    auto load_q = [&](const Unit& x, bool live, bf16x8 (&qf)[KS]) {
        const bf16x8* qh = qfrag + (((long)x.b * p.H + x.h) * nbt + nbc) * KS * kWave + (live ? lane : 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = qh[live ? ks * kWave : 0];
    };
    // folded row statistic of this lane's text row for the unit's head (-inf beyond txt_len)
    auto load_c = [&](const Unit& x) -> float {
        const float c = cstat[((long)x.b * p.H + x.h) * p.Npad + i];
        return has_rows ? c : -INFINITY;
    };
    auto frags = [&](int slot, int kt, bf16x8 (&f)[KS]) {
        const char* q = s_k + slot * SLOT_BYTES + ((tw * KT + kt) * 32 + (lane & 31)) * PITCH + (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(q + ks * 32);
    };
    auto add_probs = [&](f32x16& a, const f32x16& acc, float c) {
#pragma unroll
        for (int r = 0; r < 16; ++r) a[r] += fast_exp2(fmaf(acc[r], scale_log2e, c));
    };

    f32x16 a_acc[KT];
    auto clear_acc = [&]() {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) a_acc[kt][r] = 0.f;
    };
    // the piece of key group (x.b, x.kg) this block holds: apart[piece][b][j][i], text rows contiguous
    auto flush = [&](const Unit& x) {
        const int piece = pb - unit_block((long)x.t * p.H, P, U);
        if (has_rows) {
            float* ap = apart + (((long)piece * p.B + x.b) * p.Mv) * p.Npad + i;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = x.kg * KB + (tw * KT + kt) * 32 + tile_row(r, lane);
                    if (j < p.Mv) ap[(long)j * p.Npad] = a_acc[kt][r];
                }
        }
    };

    // prologue: unit u0 into slot 0, unit u0+1 in registers, fragments and statistic of unit u0
    u32x4 st[NLW];
    bf16x8 qf[KS];
    Unit xc = unit_at(u0), xq = xc, xk = xc;         // cursors: current unit, fragments, K rows
    load_k(xk, true, st);
    load_q(xq, true, qf);
    float c_cur = load_c(xq), c_nxt = 0.f;
    store_k(0, st);
    if (u0 + 1 < u1) advance(xk);
    load_k(xk, u0 + 1 < u1, st);
    clear_acc();

    // One unit.  On entry: its K rows are in `slot` (written before the barrier below), the next unit's
    // rows are in `st`, its fragments in qf.  The fragments of the next unit replace them as soon as the
    // last MFMA chain of this unit is under way.
    auto unit_step = [&](long u, int slot) {
        __syncthreads();                              // slot is complete; the other slot is no longer read
        store_k(slot ^ 1, st);                        // unit u+1
        if (u + 2 < u1) advance(xk);
        load_k(xk, u + 2 < u1, st);                   // unit u+2
        if (u + 1 < u1) advance(xq);
        c_nxt = load_c(xq);
        bf16x8 kfA[KS], kfB[KS];
        f32x16 accA, accB;
        frags(slot, 0, kfA);
        if constexpr (KT > 1) frags(slot, 1, kfB);
        accA = score_tile<KS>(kfA, qf);
#pragma unroll
        for (int kt = 1; kt < KT; ++kt) {
            // the MFMA chain of tile kt together with the exp2 work of tile kt-1
            if (kt & 1) {
                accB = score_tile<KS>(kfB, qf);
                if (kt + 1 < KT) frags(slot, kt + 1, kfA);
                add_probs(a_acc[kt - 1], accA, c_cur);
            } else {
                accA = score_tile<KS>(kfA, qf);
                if (kt + 1 < KT) frags(slot, kt + 1, kfB);
                add_probs(a_acc[kt - 1], accB, c_cur);
            }
        }
        load_q(xq, u + 1 < u1, qf);                   // unit u+1
        add_probs(a_acc[KT - 1], ((KT - 1) & 1) ? accB : accA, c_cur);
        c_cur = c_nxt;
        if (xc.h == p.H - 1 || u + 1 == u1) {         // the run leaves this key group
            flush(xc);
            clear_acc();
        }
        advance(xc);
    };
    long u = u0;
    for (; u + 1 < u1; u += 2) {
        unit_step(u, 0);
        unit_step(u + 1, 1);
    }
    if (u < u1) unit_step(u, 0);
}

// Column statistics (Eq. 8 / Eq. 10): a[i][j] = sum over the pieces of j's key group (fixed order);
// V_j = sum_i a[i][j], I_j = max_i a[i][j].  A wave takes four neighbouring vision keys at a time (same
// key group, same pieces), lanes over text rows; all loads of a piece are in flight together.
constexpr int kFixKeys = 4;
__global__ __launch_bounds__(256) void prefill_colfix_kernel(
    const float* __restrict__ apart, const uint8_t* __restrict__ vis_valid, const int32_t* __restrict__ mv_eff,
    PrefillDims p, ColPlan cp, float* __restrict__ Vout, float* __restrict__ Iout)
{
    const int lane = lane_id(), wv = wave_id(), b = blockIdx.y;
    const long gstride = (long)p.B * p.Mv * p.Npad;
    const int j0 = (blockIdx.x * 4 + wv) * kFixKeys;
    if (j0 >= p.Mv) return;
    const ColRun run = effective_run(mv_eff, p.B, p.H, cp, b);
    // keys behind the rows that matter: no pieces were written, their scores are zero
    const bool skipped = j0 / cp.kb >= run.nk;
    const long tile = run.tile0 + j0 / cp.kb;
    const int npieces = skipped ? 0 : unit_block(tile * p.H + p.H - 1, run.P, run.U) - unit_block(tile * p.H, run.P, run.U) + 1;
    float s[kFixKeys], mx[kFixKeys];
#pragma unroll
    for (int q = 0; q < kFixKeys; ++q) { s[q] = 0.f; mx[q] = 0.f; }
    for (int i0 = 0; i0 < p.Npad; i0 += 2 * kWave) {
        // two text rows per lane and round (lanes beyond Npad read a valid row and drop it)
        const int ia = i0 + lane, ib = i0 + kWave + lane;
        const bool oka = ia < p.Npad, okb = ib < p.Npad;
        const int ca = oka ? ia : 0, cb = okb ? ib : 0;
        float a0[kFixKeys], a1[kFixKeys];
#pragma unroll
        for (int q = 0; q < kFixKeys; ++q) { a0[q] = 0.f; a1[q] = 0.f; }
        for (int g = 0; g < npieces; ++g) {
            float x0[kFixKeys], x1[kFixKeys];
#pragma unroll
            for (int q = 0; q < kFixKeys; ++q) {
                const float* ap = apart + g * gstride + ((long)b * p.Mv + min(j0 + q, p.Mv - 1)) * p.Npad;
                x0[q] = __builtin_nontemporal_load(ap + ca);       // a piece is read once
                x1[q] = __builtin_nontemporal_load(ap + cb);
            }
#pragma unroll
            for (int q = 0; q < kFixKeys; ++q) { a0[q] += x0[q]; a1[q] += x1[q]; }
        }
#pragma unroll
        for (int q = 0; q < kFixKeys; ++q) {
            const float v0 = oka ? a0[q] : 0.f, v1 = okb ? a1[q] : 0.f;
            s[q] += v0 + v1;
            mx[q] = fmaxf(mx[q], fmaxf(v0, v1));
        }
    }
#pragma unroll
    for (int q = 0; q < kFixKeys; ++q) {
        const float ss = wave_sum(s[q]), mm = wave_max(mx[q]);
        const int j = j0 + q;
        if (lane == 0 && j < p.Mv) {
            const bool ok = !vis_valid || vis_valid[(long)b * p.Mv + j];
            Vout[(long)b * p.Mv + j] = ok ? ss : 0.f;
            Iout[(long)b * p.Mv + j] = ok ? mm : 0.f;
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
        __builtin_nontemporal_store(a2, tr.v_out + dst * kv + c);          // streaming stores: see prefill_compact_kernel
    }
    for (int c = c0; c < hv; c += 256)
        __builtin_nontemporal_store(__builtin_nontemporal_load(tr.hidden + src * hv + c), tr.hidden_out + dst * hv + c);
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
    __shared__ int s_hist[kSelectHistInts];
    if ((int)blockIdx.x >= p.B) {                    // block-uniform: the blocks that copy the text rows
        copy_text_rows<IPT>(p, tr, vis_valid, txt_len, is_key, budget, s_red);
        return;
    }
    const int b = blockIdx.x, tid = threadIdx.x;
    if (tid < 256) s_hist[tid] = 0;                  // for block_select_topk, after later barriers
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
        const SelectBound sb = block_select_topk<IPT>(rk, extra, s_hist);
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
    // hidden and V rows are written with streaming stores: nothing on this path reads them again, and left as
    // dirty lines in the Infinity Cache they would be written back in the middle of whatever kernel streams
    // through it next (measured: the sweep that follows 150 MB of plain stores takes 10 us longer); the K
    // rows, which a scoring pass reads next, keep plain stores
    auto put = [](u32x4* q, const u32x4& v, bool nt) { if (nt) __builtin_nontemporal_store(v, q); else *q = v; };
    auto copy2 = [&](const u32x4* __restrict__ s0, u32x4* __restrict__ d0, const u32x4* __restrict__ s1,
                     u32x4* __restrict__ d1, int n, bool nt0, bool nt1) {
        const int step = 2 * blockDim.x;
        for (int c = threadIdx.x; c < n; c += step) {
            const int c2 = c + blockDim.x;
            const bool two = c2 < n;
            const u32x4 a0 = __builtin_nontemporal_load(s0 + c), a1 = __builtin_nontemporal_load(s1 + c);
            u32x4 b0 = a0, b1 = a1;
            if (two) { b0 = __builtin_nontemporal_load(s0 + c2); b1 = __builtin_nontemporal_load(s1 + c2); }
            put(d0 + c, a0, nt0);
            put(d1 + c, a1, nt1);
            if (two) { put(d0 + c2, b0, nt0); put(d1 + c2, b1, nt1); }
        }
    };
    copy2(ks, kd, vs, vd, kv, false, true);
    const int half = (hv + 1) / 2;                   // the hidden row as two halves
    copy2(hs, hd, hs + half, hd + half, hv - half, true, true);
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

struct PrefillWorkspace {
    float2* partial; float* cstat; bf16x8* qfrag; float* apart; float* V; float* I; float* score; int32_t* src_row;
    int32_t* mv_eff;
    size_t bytes;
};

#ifndef MD_RS_BLOCKS
#define MD_RS_BLOCKS 512   // target number of blocks of the row-statistics sweep (two per CU)
#endif


// Launch shapes of the two sweeps; pure host arithmetic shared by the workspace size and the launch.
struct ScorePlan { int nbt, nbw, ng, nch, chunk, rs_waves; ColPlan col; int occ; };
constexpr int kNumCU = 256;                          // MI355X

ScorePlan plan_scores(int B, int Mv, int N, int H) {
    ScorePlan s;
    s.nbt = (N + 31) / 32;                            // 32-row text blocks
    s.nbw = s.nbt == 1 ? 1 : (s.nbt == 2 ? 2 : 4);    // text blocks per block (one per wave or wave pair)
    s.ng = (s.nbt + s.nbw - 1) / s.nbw;               // text groups: K is read once per group
    // sweep 1: chunks of whole 128-key units, enough blocks to fill the chip a few times, at least
    // four units per chunk
    const int units = (Mv + N + 127) / 128;
    int nch = (MD_RS_BLOCKS + B * H * s.ng - 1) / (B * H * s.ng);
    // four text blocks and two chunks per (sample, head): one block of eight waves takes both halves instead
    // (same number of waves on the chip, the halves' statistics meet in LDS, no merge kernel)
    s.rs_waves = 4;
    if (s.nbw == 4 && nch == 2) { s.rs_waves = 8; nch = 1; }
    if (nch > units / 4) nch = units / 4;
    if (nch < 1) nch = 1;
    if (nch > kMaxChunks) nch = kMaxChunks;
    const int upc = (units + nch - 1) / nch;
    s.chunk = upc * 128;
    s.nch = (units + upc - 1) / upc;
    // sweep 2: a persistent grid; units of (kb keys, one head), at least four per block
    ColPlan& c = s.col;
    c.kb = s.nbw == 1 ? 128 : 64;
    c.nkg = (Mv + c.kb - 1) / c.kb;
    c.U = (long)B * c.nkg * H;
    // blocks per CU: two where a block holds four text blocks (the second block covers the first one's waits),
    // and with two text blocks when the runs stay long enough (20 units per CU); otherwise one (fewer, longer
    // runs: fewer pieces, fewer prologues; measured faster there)
    s.occ = s.nbw == 4 || (s.nbw == 2 && c.U >= 20L * kNumCU) ? 2 : 1;
    long P = (c.U + 3) / 4;
    if (P > kNumCU * s.occ) P = kNumCU * s.occ;
    if (P < 1) P = 1;
    c.P = (int)P;
    // pieces a key group can be cut into; sized for half the planned units (samples whose valid vision rows
    // are a prefix of their slots bring fewer key groups), beyond that fewer blocks work
    c.Gmax = (int)((2L * H * c.P + c.U - 1) / c.U) + 1;
    if (c.Gmax > H) c.Gmax = H;
    return s;
}

PrefillWorkspace carve_prefill(void* base, int B, int Mv, int N, int H, int Rcap) {
    Carver c(base);
    PrefillWorkspace w;
    const ScorePlan s = plan_scores(B, Mv, N, H);
    const int Npad = s.nbt * 32;
    w.partial = c.take<float2>((size_t)B * H * s.nch * Npad);
    w.cstat = c.take<float>((size_t)B * H * Npad);
    w.qfrag = c.take<bf16x8>((size_t)B * H * Npad * 16);      // [B][H][NB][KS][64] fragments, d <= 128
    w.apart = c.take<float>((size_t)s.col.Gmax * B * Mv * Npad);
    w.V = c.take<float>((size_t)B * Mv);
    w.I = c.take<float>((size_t)B * Mv);
    w.score = c.take<float>((size_t)B * Mv);
    w.src_row = c.take<int32_t>((size_t)B * (Rcap + N));
    w.mv_eff = c.take<int32_t>((size_t)B);
    w.bytes = c.off;
    return w;
}

template <int KS>
int launch_scores(const PrefillDims& p, const ScorePlan& s, const PrefillWorkspace& w, hipStream_t st, const void* q_txt,
                  const void* k, const uint8_t* vis_valid, const int32_t* txt_len, const float* row_lse, float scale_log2e) {
    const uint16_t* qp = static_cast<const uint16_t*>(q_txt);
    const uint16_t* kp = static_cast<const uint16_t*>(k);
    if (!row_lse) {
        dim3 g1(p.nch * s.ng, p.H, p.B);
#define MD_ROWSTATS(NBW_, TW_)                                                                                 \
        MD_LAUNCH("prefill_rowstats", st, (prefill_rowstats_kernel<NBW_, TW_, KS>), g1, 64 * NBW_ * TW_, 0,   \
            qp, kp, vis_valid, txt_len, p, scale_log2e, w.partial, w.cstat, w.qfrag, w.mv_eff)
        if (s.nbw == 1) MD_ROWSTATS(1, 4);
        else if (s.nbw == 2) MD_ROWSTATS(2, 2);
        else if (s.rs_waves == 8) MD_ROWSTATS(4, 2);
        else MD_ROWSTATS(4, 1);
#undef MD_ROWSTATS
        if (p.nch > 1) {
            const long n = (long)p.B * p.H * p.Npad;
            MD_LAUNCH("prefill_cstat", st, (prefill_cstat_kernel), (unsigned)((n + 255) / 256), 256, 0, w.partial, txt_len, p, w.cstat);
        }
    } else {
        const long items = (long)p.B * p.H * s.nbt;
        MD_LAUNCH("prefill_qpack", st, (prefill_qpack_kernel<KS>), (unsigned)((items + 3) / 4 + p.B), 256, 0, qp, vis_valid, txt_len,
                  row_lse, p, w.qfrag, w.cstat, w.mv_eff);
    }
    for (int tg = 0; tg < s.ng; ++tg) {
#define MD_COLSCORE(NBW_, KT_)                                                                                 \
        MD_LAUNCH("prefill_colscore", st, (prefill_colscore_kernel<NBW_, KT_, KS>), s.col.P, 256, 0,           \
            w.qfrag, kp, w.cstat, w.mv_eff, p, s.col, scale_log2e, tg, w.apart)
        // 32 * (4 / NBW) * KT keys per unit = s.col.kb
        if (s.nbw == 1) MD_COLSCORE(1, 1);
        else if (s.nbw == 2) MD_COLSCORE(2, 1);
        else MD_COLSCORE(4, 2);
#undef MD_COLSCORE
    }
    const int fx = (p.Mv + 4 * kFixKeys - 1) / (4 * kFixKeys);          // four waves of kFixKeys keys per block
    MD_LAUNCH("prefill_colfix", st, (prefill_colfix_kernel), dim3(fx, p.B), 256, 0, w.apart, vis_valid, w.mv_eff, p, s.col, w.V, w.I);
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
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key, const float* row_lse,
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
    // the score sweeps address a sample's head slice with 32-bit byte offsets
    if (((long)L * lkv.token + d) * 2 >= (1l << 31) || ((long)N * lq.token + d) * 2 >= (1l << 31))
        return fail(MD_ESHAPE, "prefill_filter: one head slice of a sample spans more than 2 GiB");
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
    const ScorePlan sp = plan_scores(B, Mv, N, H);
    p.Npad = sp.nbt * 32;
    p.nch = sp.nch; p.chunk = sp.chunk;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float sl2 = softmax_scale * kLog2e;

    int rc = d == 128 ? launch_scores<8>(p, sp, w, st, q_txt, k, vis_valid, txt_len, row_lse, sl2)
                      : launch_scores<4>(p, sp, w, st, q_txt, k, vis_valid, txt_len, row_lse, sl2);
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
    else if (Mv <= 3072) MD_PSELECT_FAST(3);
    else if (Mv <= 4096) MD_PSELECT_FAST(4);
    else if (Mv <= 5120) MD_PSELECT_FAST(5);
    else if (Mv <= 6144) MD_PSELECT_FAST(6);
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
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key, const float* row_lse,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return prefill_filter_impl(q_txt, k, v, hidden, vis_valid, txt_len, is_key, row_lse, B, Mv, N, H, d, C, softmax_scale, mode,
                               budget, gamma, alpha, Rcap, hidden_out, k_out, v_out, kept_index, kept_count, out_len,
                               out_protect, out_ids, score_global, score_indiv, nullptr, nullptr, nullptr,
                               workspace, workspace_bytes, stream);
}

extern "C" int mustdrop_prefill_filter_strided(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key, const float* row_lse,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    const md_kv_layout* q_layout, const md_kv_layout* kv_layout, const md_kv_layout* kv_out_layout,
    void* workspace, size_t workspace_bytes, void* stream)
{
    return prefill_filter_impl(q_txt, k, v, hidden, vis_valid, txt_len, is_key, row_lse, B, Mv, N, H, d, C, softmax_scale, mode,
                               budget, gamma, alpha, Rcap, hidden_out, k_out, v_out, kept_index, kept_count, out_len,
                               out_protect, out_ids, score_global, score_indiv, q_layout, kv_layout, kv_out_layout,
                               workspace, workspace_bytes, stream);
}
