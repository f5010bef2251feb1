/*
 * mustdrop.h -- C ABI of the MustDrop token-reduction library for AMD MI355X (gfx950).
 *
 * Three entry points, one per stage of the method (Liu et al., "Multi-Stage
 * Vision Token Dropping", CVPR 2025):
 *   mustdrop_encode_merge    Sec. 3.3  Local Spatial Merging (Eq. 5) + Key Retaining (Eq. 6-7)
 *   mustdrop_prefill_filter  Sec. 3.4  dual-attention filtering (Eq. 8-10) + token drop
 *   mustdrop_decode_evict    Sec. 3.5  output-aware cache policy, one decode step
 *
 * Conventions common to all calls
 *   - Every data pointer is DEVICE memory owned by the caller (inputs, outputs and the workspace).
 *     The entry points of this header allocate nothing, free nothing and keep no state between
 *     calls, with these exceptions, all stated here: the thread-local text behind
 *     mustdrop_last_error(); the static device buffer of mustdrop_encode_merge_noalloc and the
 *     address of it that the library looks up once per device (see there); and, while a caller
 *     has switched on the benchmarking aid declared in mustdrop_bench.h (a separate header, not
 *     needed to use the method), one pair of HIP events per kernel launch.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream).  No
 *     call synchronises with the host; variable-length results are reported through device-side
 *     count arrays and the outputs are padded to a static capacity.
 *   - Tensors are row-major with the last dimension contiguous.  Base pointers of the large
 *     tensors must be 16-byte aligned and their rows (D, dc, d, C elements) a multiple of 16 bytes.
 *   - Indices are int32, 0-based, in the coordinates of that call's input; index lists ascend.
 *   - Inputs are never written, except the in/out state of mustdrop_decode_evict.
 *   - Return value: MD_OK or an error code.  Argument errors are detected on the host before any
 *     kernel is launched; mustdrop_last_error() returns a thread-local description.
 *   - `workspace` must hold at least mustdrop_<stage>_workspace_bytes(...) bytes, 256-byte aligned.
 *     Calls that share a workspace must be ordered on one stream.  Calls that share neither a
 *     workspace nor an output or state buffer may overlap in time (several streams): a caller with
 *     independent batches can keep two of them in flight.
 */
#ifndef MUSTDROP_H
#define MUSTDROP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types and modes cross the boundary as plain ints (a caller may hand over any value: one
 * that names nothing is an error code, never undefined behaviour). */
typedef int md_dtype;
enum { MD_F32 = 0, MD_BF16 = 1 };

typedef enum {
    MD_OK = 0,
    MD_EINVAL = 1,      /* null required pointer, non-positive size, value out of range */
    MD_ESHAPE = 2,      /* shapes that do not fit together or that no kernel supports   */
    MD_EALIGN = 3,      /* pointer or row size not 16-byte aligned                      */
    MD_EALIAS = 4,      /* an output overlaps an input                                  */
    MD_EWORKSPACE = 5,  /* workspace missing or too small                               */
    MD_EDTYPE = 6,      /* unknown dtype / mode enum                                    */
    MD_EHIP = 7         /* the HIP runtime reported an error at launch                  */
} md_status;

typedef int md_filter_mode;
enum { MD_FILTER_BUDGET = 0, MD_FILTER_THRESHOLD = 1 };

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* mustdrop_last_error(void);

/* Library version, major*100 + minor (2: mustdrop_prefill_filter takes row_lse). */
int mustdrop_version(void);

/* ------------------------------------------------------------------------------------------
 * Stage 1 -- vision encoding (Sec. 3.3).
 *
 * Key Retaining (Eq. 6-7): a_cls[j] = mean over the Hc heads of softmax_j(q_cls . k_j / sqrt(dc)),
 * the softmax running over all 1+M keys (key 0 is the [CLS] key, whose own probability is
 * discarded).  The key set O is the `key_budget` valid tokens with the largest a_cls (ties: lower
 * index).  Local Spatial Merging (Eq. 5): the T x Hg x Wg grid is cut into non-overlapping
 * kt x kh x kw windows (where the window does not divide the grid, the windows at the far border are
 * clipped to the grid and hold fewer tokens); S = mean over unordered member pairs of their cosine
 * similarity (zero-norm member: cosine 0).  A window merges iff S > tau, it has at least two valid members and none of
 * them is in O; its members are replaced by one token: the mass-weighted mean of the members, with
 * mass = sum of member masses, at the position of the lowest member index.  Survivors are written
 * in ascending original index.
 *
 *   x          [B, M, D]          M = T*Hg*Wg, token index = (t*Hg + y)*Wg + x; dtype x_dtype
 *   q_cls      [B, Hc, dc]        CLS query;   k_cls [B, 1+M, Hc, dc] keys (row 0 = CLS key);
 *                                 dtype qk_dtype; both NULL iff key_budget == 0; dc a power of two
 *   mass_in    [B, M] f32 or NULL (all ones)      valid [B, M] u8 or NULL (all valid)
 *   tau        threshold on the MEAN pairwise cosine (the paper's ordered-pair sum is
 *              ws*(ws-1) times the mean, ws = kt*kh*kw)
 *   out_x      [B, M, D]  dtype x_dtype; rows >= out_count[b] are left untouched.  Unmerged rows
 *              are bit-identical copies; merged rows are accumulated in fp32 and rounded to nearest even
 *   out_index, out_mass, out_is_key [B, M]; out_valid [B, M] u8 (1 for slots < out_count[b]; may be NULL)
 *   out_count  [B]
 *   key_index  [B, key_budget] ascending, padded with -1 if fewer valid tokens exist
 *   a_cls_out  [B, M] f32 or NULL;  window_sim_out [B, W] f32 or NULL,
 *              W = ceil(T/kt)*ceil(Hg/kh)*ceil(Wg/kw), window index = (wt*ceil(Hg/kh) + wy)*ceil(Wg/kw) + wx
 *
 * Limits: kt*kh*kw <= 16; D*elt and dc*elt multiples of 16 bytes.
 * Errors: MD_EINVAL, MD_ESHAPE (window too large, Hc*dc unusable), MD_EALIGN, MD_EALIAS (out_x overlaps x), MD_EWORKSPACE, MD_EDTYPE, MD_EHIP.
 */
size_t mustdrop_encode_merge_workspace_bytes(int B, int T, int Hg, int Wg, int Hc, int kt, int kh, int kw);

int mustdrop_encode_merge(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_budget,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index,
    float* a_cls_out, float* window_sim_out,
    void* workspace, size_t workspace_bytes, void* stream);

/* mustdrop_encode_merge for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * errors as mustdrop_encode_merge, minus `workspace` / `workspace_bytes`: the scratch memory is a static
 * device array of MUSTDROP_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds
 * one until the process ends).  The call allocates and frees nothing.  A shape whose
 * mustdrop_encode_merge_workspace_bytes(...) exceeds the static buffer is rejected with MD_EWORKSPACE
 * (8 MiB covers up to 16 samples of 2880 tokens, or 4 of 4608, with 16 CLS heads).  The first call on
 * a device looks up the array's device address; do that call outside a graph capture.  All calls on one
 * GPU share the array, which keeps the previous call's contents (nothing in it needs clearing): calls
 * that overlap in time on one GPU race -- order them on one stream. */
#define MUSTDROP_STATIC_SCRATCH_BYTES (8u << 20)

int mustdrop_encode_merge_noalloc(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_budget,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index,
    float* a_cls_out, float* window_sim_out, void* stream);

/* Stage 1 with the key set in the printed form of Eq. 7: O = { j : a_cls[j] > mu }.  The paper only says
 * that mu is adaptive and depends on a_cls; this library reads it as mu = mean + key_lambda * std of
 * a_cls over the valid tokens (population standard deviation, fp32).  Everything else is
 * mustdrop_encode_merge.  key_cap >= 0 is the capacity of key_index per sample ([B, key_cap], may be
 * NULL if 0): the first key_cap members of O in ascending order, the rest -1; key_count [B] (required)
 * receives |O|, which may exceed key_cap.  q_cls and k_cls are always required. */
int mustdrop_encode_merge_adaptive(
    const void* x, md_dtype x_dtype,
    const void* q_cls, const void* k_cls, md_dtype qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, float key_lambda, int key_cap,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key, uint8_t* out_valid,
    int32_t* out_count, int32_t* key_index, int32_t* key_count,
    float* a_cls_out, float* window_sim_out,
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Stage 2 -- prefill, one LLM layer (Sec. 3.4).  Sequence per sample: [vision 0..Mv-1 | text 0..N-1]
 * (Sec. 3.1, prefilling: X = {V_1..V_M, T_1..T_N}), L = Mv + N.
 *
 * a[i][j] = mean over heads of the softmax probability of text row i on vision column j; each
 * text row's softmax runs over the valid vision keys and the text keys 0..i (causal).
 * V_j = sum_i a[i][j] (Eq. 8), I_j = max_i a[i][j] (Eq. 10), G = sum_j V_j (Eq. 9, valid j only).
 *   MD_FILTER_THRESHOLD: drop j iff V_j <= gamma*G and I_j < alpha and j is not a key token.
 *   MD_FILTER_BUDGET:    keep the key tokens, then the (budget - #keys) other valid tokens with
 *                        the largest s_j = max(V_j/(gamma*G), I_j/alpha) (ties: lower index);
 *                        gamma, alpha > 0 required.
 * Token drop: rows [kept vision tokens ascending | text rows 0..txt_len-1] of hidden, k and v are
 * copied bit for bit to the outputs.
 *
 *   q_txt      [B, N, H, d] bf16   queries of the text tokens
 *   k, v       [B, L, H, d] bf16;  hidden [B, L, C] bf16
 *   vis_valid  [B, Mv] u8 or NULL; txt_len [B] i32 or NULL (= N; text is padded at the tail);
 *   is_key     [B, Mv] u8 or NULL (no key tokens)
 *   row_lse    [B, H, N] f32 or NULL.  The scores a[i][j] are a by-product of the layer's own attention
 *              (Sec. 3.4); a flash-style attention kernel keeps, per head and query row, the natural-log
 *              sum of exp(softmax_scale * q.k) over the keys that row sees.  Given those values for the text rows
 *              (over the valid vision keys and the text keys 0..i, with this call's softmax_scale), the
 *              library skips its own pass over K for the softmax normalisers and reads K once instead
 *              of twice.  Entries of rows >= txt_len are ignored.  NULL: the library computes them.
 *   Rcap       capacity, in rows, of the kept-vision part of the outputs (>= budget in budget mode;
 *              use Mv in threshold mode).  The caller must size it for max(budget, #keys).
 *   hidden_out [B, Rcap+N, C], k_out, v_out [B, Rcap+N, H, d]; rows >= out_len[b] untouched
 *   kept_index [B, Rcap] (entries >= min(kept_count, Rcap) untouched)
 *   kept_count [B]   number of vision tokens the rule keeps; if it exceeds Rcap only the first
 *                    Rcap (lowest indices) are stored -- an overflow the caller can detect
 *   out_len    [B] or NULL   = min(kept_count, Rcap) + txt_len: live rows of the outputs
 *   out_ids    [B, Rcap+N] i32 or NULL: original sequence position of every output row (vision index j,
 *              or Mv+i for text row i; -1 for rows that are not live) -- usable as the decode stage's ids
 *   out_protect[B, Rcap+N] u8 or NULL: 1 for key tokens and text rows (the decode stage's protect flags)
 *   score_global, score_indiv [B, Mv] f32 or NULL: V_j and I_j (0 for invalid tokens)
 *
 * Limits: d in {64, 128}; N <= 1024 (tuned for N <= 128: a longer prompt re-reads K once per 64
 * text rows in the first sweep and once per 128 in the second); H <= 128; softmax_scale positive
 * and finite; C*2 and H*d*2 multiples of 16 bytes.
 */
size_t mustdrop_prefill_filter_workspace_bytes(int B, int Mv, int N, int H, int Rcap);

int mustdrop_prefill_filter(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key, const float* row_lse,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Stage 3 -- decode, one step of one layer (Sec. 3.5; decode attention as in Eq. 4).
 *
 * a_t[j] = mean over heads of softmax_j(softmax_scale * q_h . k_jh) over the live entries
 * j < len[b]; acc[j] <- decay*acc[j] + a_t[j].  If len[b] > budget, the protected entries and the
 * (budget - #protected) unprotected entries with the largest acc stay (ties: lower id); the rest
 * are evicted.  With protect = the set S_few and budget = |S_few| this is the paper's static
 * policy.  The cache is compacted by hole filling: survivors sitting at slots >= new_len move, in
 * ascending slot order, into the evicted slots < new_len, in ascending slot order; K/V rows move
 * bit for bit together with their acc / ids / protect entries.
 *
 *   q        [B, H, d] bf16             query of the token being generated
 *   k_cache, v_cache [B, Lcap, H, d] bf16   in/out
 *   acc      [B, Lcap] f32 (>= 0: entries are ranked by the bit pattern of their score), ids [B, Lcap] i32
 *            (in [0, 2^31 - 2], unique per sample), protect [B, Lcap] u8, len [B] i32: in/out
 *   decay    >= 0 (MD_EINVAL otherwise), so that the running scores stay non-negative
 *   evicted_ids [B, Lcap] or NULL: ids of the evicted entries in ascending (pre-compaction) slot order
 *   evicted_count [B] or NULL
 *
 * Limits: d a power of two in [8, 512]; H <= 1024 (rows of 1, 2, 4 or 8 KiB with d = 128 and
 * H in {4, 8, 16, 32, 64} take the streaming kernels, other shapes the general ones).
 * MD_EALIAS: q, the two caches, acc, ids, protect, len, the optional outputs and the workspace must be
 * pairwise disjoint.
 */
size_t mustdrop_decode_evict_workspace_bytes(int B, int Lcap, int H);

int mustdrop_decode_evict(
    const void* q, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d,
    float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count,
    void* workspace, size_t workspace_bytes, void* stream);

/* Appends one entry per sample at slot len[b] (Eq. 3: K <- Concat(K, x_i W_k), same for V):
 * copies k_new[b], v_new[b] ([B, H, d] bf16), sets acc = 0, ids = new_id, protect = protect_new,
 * len[b] += 1.  Samples whose cache is full (len[b] == Lcap) are left unchanged.  Device-side,
 * asynchronous, so a decode loop needs no host round trip. */
int mustdrop_decode_append(
    const void* k_new, const void* v_new,
    void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, int32_t new_id, int protect_new, void* stream);

/* ------------------------------------------------------------------------------------------
 * Stage 3, the static policy as printed (Sec. 3.5): from the shallow layers on, the caches store only
 * the vision tokens of the set S_few (besides the text and what was generated) -- nothing is scored.
 * keep[b][j] != 0 marks the entries j < len[b] that stay.  The caches of all n_layers layers are
 * compacted in one call by the hole filling of mustdrop_decode_evict (the kept entries at slots
 * >= new_len move, in ascending order, into the dropped slots < new_len, in ascending order), so every
 * layer holds the same entry in the same slot and ids / protect / acc describe all of them.
 *
 *   k_cache, v_cache [n_layers, B, Lcap, H, d] bf16, in/out (device)
 *   keep     [B, Lcap] u8, read only (entries >= len[b] are ignored)
 *   acc      [B, Lcap] f32 in/out, or NULL;  ids [B, Lcap] i32, protect [B, Lcap] u8, len [B] i32: in/out
 *   evicted_ids [B, Lcap] or NULL: ids of the dropped entries in ascending slot order;
 *   evicted_count [B] or NULL
 *   workspace: mustdrop_decode_evict_workspace_bytes(B, Lcap, H) bytes, 256-byte aligned
 * Limits and errors as for mustdrop_decode_evict; n_layers in [1, 65535].
 */
int mustdrop_decode_keep(
    void* k_cache, void* v_cache, const uint8_t* keep,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d,
    int32_t* evicted_ids, int32_t* evicted_count,
    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Other memory layouts of Q, K and V (the tensors of Eq. 3-4; what the stages compute is unchanged).
 *
 * The entry points above take the token-major layout [B, tokens, H, d].  The *_strided twins below
 * take, per tensor group, the ELEMENT strides of the batch, token and head axes; the d elements of
 * one (sample, token, head) stay contiguous.  A head-major cache [B, H, tokens, d] is
 * {H*tokens*d, d, tokens*d}; a token-major one with padded rows {tokens*pitch, pitch, d}.
 * A NULL layout means dense token-major, and a call whose layouts are all dense token-major takes
 * exactly the path of the plain entry point.  For other layouts the score kernels run with strided
 * addressing and the row copies gather a token's row head slice by head slice (d*2 contiguous
 * bytes at a time).
 *
 * Every stride must be a positive multiple of 8 elements (16 bytes), and the three axes must nest
 * without overlap: sorted by stride, stride[0] >= d, stride[1] >= stride[0]*extent[0],
 * stride[2] >= stride[1]*extent[1] (else MD_ESHAPE).  The caller's allocation must cover
 * (B-1)*batch + (tokens-1)*token + (H-1)*head + d elements from the base pointer.
 * All other arguments, outputs, limits and errors are those of the plain entry point.
 */
typedef struct {
    int64_t batch;   /* elements between consecutive samples       */
    int64_t token;   /* elements between consecutive tokens/slots  */
    int64_t head;    /* elements between consecutive heads         */
} md_kv_layout;      /* host memory; read during the call only     */

/* q_layout: q_txt over N tokens; kv_layout: k and v over L = Mv+N tokens (one layout for both);
 * kv_out_layout: k_out and v_out over Rcap+N rows.  hidden and hidden_out stay [B, rows, C]. */
int mustdrop_prefill_filter_strided(
    const void* q_txt, const void* k, const void* v, const void* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key, const float* row_lse,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, md_filter_mode mode, int budget, float gamma, float alpha,
    int Rcap,
    void* hidden_out, void* k_out, void* v_out,
    int32_t* kept_index, int32_t* kept_count, int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    float* score_global, float* score_indiv,
    const md_kv_layout* q_layout, const md_kv_layout* kv_layout, const md_kv_layout* kv_out_layout,
    void* workspace, size_t workspace_bytes, void* stream);

/* cache_layout: k_cache and v_cache over Lcap slots.  q, k_new, v_new stay [B, H, d]. */
int mustdrop_decode_evict_strided(
    const void* q, void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d,
    float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count,
    const md_kv_layout* cache_layout,
    void* workspace, size_t workspace_bytes, void* stream);

int mustdrop_decode_append_strided(
    const void* k_new, const void* v_new,
    void* k_cache, void* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d, int32_t new_id, int protect_new,
    const md_kv_layout* cache_layout, void* stream);

/* layer_stride: elements between the caches of consecutive layers (ignored when n_layers == 1;
 * a positive multiple of 8 that is at least the extent of one layer's cache, else MD_ESHAPE). */
int mustdrop_decode_keep_strided(
    void* k_cache, void* v_cache, const uint8_t* keep,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d,
    int32_t* evicted_ids, int32_t* evicted_count,
    const md_kv_layout* cache_layout, int64_t layer_stride,
    void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MUSTDROP_H */
