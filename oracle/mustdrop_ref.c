/*
 * CPU oracle for the MustDrop token-reduction path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of the three stages exactly as the paper
 * states them (Sec. 3.3 Eq. 5-7, Sec. 3.4 Eq. 8-10, Sec. 3.5), with the
 * readings listed in the design notes where the text is silent.  It shares no
 * code with the HIP library, is never linked into it, and is only called from
 * the tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * Everything is nested loops over host pointers.  Stored inputs (fp32 or bf16
 * bit patterns) are widened exactly to double; values stored in an input dtype
 * are rounded once, to nearest even, from the double result.
 *
 * Pins (tests/test_oracle_*.py): closed forms (constant image, orthogonal
 * tokens, zero queries -> harmonic numbers), conservation of token mass,
 * brute-force enumeration on tiny grids, an independent numpy einsum+softmax,
 * stable-argsort selection, subset brute force for eviction, a direct
 * construction of the hole-filling layout over several layers, and the figures
 * printed in Tables 1 and 3 (tests/test_golden.py).  Parity unpinned by
 * anything the paper prints: the numeric values of tau, mu, gamma, alpha and
 * the layer schedule (the paper defers them to an appendix that is not
 * available) -- they are caller parameters here; the form of the adaptive
 * threshold of Eq. 7 (read as mean + lambda * std; that rule itself is pinned
 * against numpy, and its strict > by an exact tie: one head, a zero CLS query
 * and 2^k - 1 tokens make every a_cls equal to mu).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_OK = 0, REF_EINVAL = 1 };
enum { REF_FILTER_BUDGET = 0, REF_FILTER_THRESHOLD = 1 };

/* ---------------------------------------------------------------- storage */
static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bf16, one rounding, ties to even (8 significant bits, min exp -126) */
static uint16_t double_to_bf16(double v) {
    if (isnan(v)) return 0x7FC0;
    if (isinf(v)) return v > 0 ? 0x7F80 : 0xFF80;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    int e;
    (void)frexp(v, &e);            /* |v| = m * 2^e, m in [0.5, 1) */
    int qe = e - 8;                /* quantum 2^qe keeps 8 significant bits */
    if (qe < -133) qe = -133;      /* subnormal bf16 quantum */
    double r = rint(ldexp(v, -qe)); /* default rounding mode: ties to even */
    double w = ldexp(r, qe);
    float f = (float)w;            /* exact, or overflow to inf */
    if (fabs(w) >= ldexp(1.0, 128)) f = v > 0 ? INFINITY : -INFINITY;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static double load_el(const void* p, int dtype, size_t i) {
    if (dtype == REF_BF16) return bf16_to_double(((const uint16_t*)p)[i]);
    return (double)((const float*)p)[i];
}

static void store_el(void* p, int dtype, size_t i, double v) {
    if (dtype == REF_BF16) ((uint16_t*)p)[i] = double_to_bf16(v);
    else ((float*)p)[i] = (float)v;
}

static size_t el_size(int dtype) { return dtype == REF_BF16 ? 2 : 4; }

/* ------------------------------------------------------- ordering helper */
typedef struct { double score; int32_t tie; int32_t slot; } ranked_t;

/* larger score first; equal scores: smaller tie value first */
static int ranked_cmp(const void* a, const void* b) {
    const ranked_t* x = (const ranked_t*)a;
    const ranked_t* y = (const ranked_t*)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    if (x->tie < y->tie) return -1;
    if (x->tie > y->tie) return 1;
    return 0;
}

/* =========================================================================
 * Stage 1 -- Sec. 3.3: Local Spatial Merging (Eq. 5) and Key Retaining
 * (Eq. 6-7, budget form).
 * ========================================================================= */
/* key_mode 0: Eq. 7 in its budget form (the key_budget largest a_cls).  key_mode 1: Eq. 7 as printed,
 * O = { a_cls > mu }, with the adaptive threshold read as mu = mean + key_lambda * std of a_cls over the
 * valid tokens (population std); key_budget is then the capacity of key_index per sample and
 * key_count[b] = |O|. */
static int encode_merge_core(
    const void* x, int x_dtype,
    const void* q_cls, const void* k_cls, int qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_mode, int key_budget, float key_lambda,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key,
    uint8_t* out_valid, int32_t* out_count, int32_t* key_index, int32_t* key_count,
    double* a_cls_out, double* window_sim_out)
{
    if (B <= 0 || T <= 0 || Hg <= 0 || Wg <= 0 || D <= 0) return REF_EINVAL;
    if (kt <= 0 || kh <= 0 || kw <= 0) return REF_EINVAL;
    const int M = T * Hg * Wg;
    if (key_budget < 0 || (key_mode == 0 && key_budget > M)) return REF_EINVAL;
    const int with_keys = key_mode == 1 || key_budget > 0;
    if (with_keys && (!q_cls || !k_cls || Hc <= 0 || dc <= 0)) return REF_EINVAL;
    if (key_mode == 1 && !key_count) return REF_EINVAL;
    const int ws = kt * kh * kw;
    /* Sec. 3.3 tiles the grid with windows of one size; where the window does not divide the grid, the
       windows at the far border are clipped to the grid and hold fewer tokens (a window left with fewer
       than two valid tokens is never merged, like any other). */
    const int nwt = (T + kt - 1) / kt, nwy = (Hg + kh - 1) / kh, nwx = (Wg + kw - 1) / kw;
    const int W = nwt * nwy * nwx;

    double* a_cls = (double*)malloc(sizeof(double) * (size_t)M);
    double* logit = (double*)malloc(sizeof(double) * (size_t)(M + 1));
    uint8_t* is_key = (uint8_t*)malloc((size_t)M);
    uint8_t* merged_tok = (uint8_t*)malloc((size_t)M);   /* token belongs to a merged window */
    int32_t* rep_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)M); /* window id if token is the representative, else -1 */
    ranked_t* order = (ranked_t*)malloc(sizeof(ranked_t) * (size_t)M);
    int* mem = (int*)malloc(sizeof(int) * (size_t)ws);
    double* mean = (double*)malloc(sizeof(double) * (size_t)D);
    uint8_t* win_merged = (uint8_t*)malloc((size_t)W);

    for (int b = 0; b < B; ++b) {
        const uint8_t* vb = valid ? valid + (size_t)b * M : NULL;
        const float* mb = mass_in ? mass_in + (size_t)b * M : NULL;

        /* ---- Key Retaining: a_cls = softmax(q_cls K^T / sqrt(d_k)) per head, head mean (Eq. 6) */
        memset(is_key, 0, (size_t)M);
        for (int j = 0; j < M; ++j) a_cls[j] = 0.0;
        if (with_keys) {
            for (int h = 0; h < Hc; ++h) {
                /* key 0 is the CLS key itself and always takes part in the softmax */
                double mx = -INFINITY;
                for (int j = 0; j <= M; ++j) {
                    if (j > 0 && vb && !vb[j - 1]) { logit[j] = -INFINITY; continue; }
                    double acc = 0.0;
                    for (int c = 0; c < dc; ++c) {
                        double qv = load_el(q_cls, qk_dtype, ((size_t)b * Hc + h) * dc + c);
                        double kv = load_el(k_cls, qk_dtype, (((size_t)b * (M + 1) + j) * Hc + h) * dc + c);
                        acc += qv * kv;
                    }
                    logit[j] = acc / sqrt((double)dc);
                    if (logit[j] > mx) mx = logit[j];
                }
                double z = 0.0;
                for (int j = 0; j <= M; ++j)
                    if (logit[j] != -INFINITY) z += exp(logit[j] - mx);
                for (int j = 1; j <= M; ++j)
                    if (logit[j] != -INFINITY) a_cls[j - 1] += exp(logit[j] - mx) / z / (double)Hc;
            }
            int nv = 0;
            for (int j = 0; j < M; ++j) {
                if (vb && !vb[j]) { a_cls[j] = -INFINITY; continue; }
                order[nv].score = a_cls[j]; order[nv].tie = j; order[nv].slot = j; ++nv;
            }
            if (key_mode == 0) {
                /* ---- key set O: the key_budget valid tokens with the largest a_cls (Eq. 7, budget form) */
                qsort(order, (size_t)nv, sizeof(ranked_t), ranked_cmp);
                int nk = key_budget < nv ? key_budget : nv;
                for (int r = 0; r < nk; ++r) is_key[order[r].slot] = 1;
            } else {
                /* ---- key set O = { a_cls > mu } (Eq. 7), mu = mean + lambda * std over the valid tokens */
                double mean_a = 0.0, var_a = 0.0;
                for (int r = 0; r < nv; ++r) mean_a += order[r].score;
                if (nv > 0) mean_a /= (double)nv;
                for (int r = 0; r < nv; ++r) var_a += (order[r].score - mean_a) * (order[r].score - mean_a);
                if (nv > 0) var_a /= (double)nv;
                const double mu = mean_a + (double)key_lambda * sqrt(var_a);
                for (int r = 0; r < nv; ++r) if (order[r].score > mu) is_key[order[r].slot] = 1;
            }
            int o = 0, total = 0;
            for (int j = 0; j < M; ++j)
                if (is_key[j]) {
                    if (o < key_budget) key_index[(size_t)b * key_budget + o++] = j;
                    ++total;
                }
            for (; o < key_budget; ++o) key_index[(size_t)b * key_budget + o] = -1;
            if (key_count) key_count[b] = total;
        } else if (key_count) key_count[b] = 0;
        if (a_cls_out) for (int j = 0; j < M; ++j) a_cls_out[(size_t)b * M + j] = a_cls[j];

        /* ---- Local Spatial Merging: mean pairwise cosine inside each window (Eq. 5) */
        memset(merged_tok, 0, (size_t)M);
        for (int j = 0; j < M; ++j) rep_of[j] = -1;
        for (int wt = 0; wt < nwt; ++wt)
        for (int wy = 0; wy < nwy; ++wy)
        for (int wx = 0; wx < nwx; ++wx) {
            const int w = (wt * nwy + wy) * nwx + wx;
            int n = 0, has_key = 0;
            for (int dt = 0; dt < kt; ++dt)
            for (int dy = 0; dy < kh; ++dy)
            for (int dx = 0; dx < kw; ++dx) {
                if (wt * kt + dt >= T || wy * kh + dy >= Hg || wx * kw + dx >= Wg) continue;   /* clipped */
                int tok = ((wt * kt + dt) * Hg + (wy * kh + dy)) * Wg + (wx * kw + dx);
                if (vb && !vb[tok]) continue;
                mem[n++] = tok;
                if (is_key[tok]) has_key = 1;
            }
            double S = 0.0;
            int npairs = 0;
            for (int m = 0; m < n; ++m)
            for (int q = m + 1; q < n; ++q) {
                double dot = 0.0, nm = 0.0, nq = 0.0;
                for (int c = 0; c < D; ++c) {
                    double xm = load_el(x, x_dtype, ((size_t)b * M + mem[m]) * D + c);
                    double xq = load_el(x, x_dtype, ((size_t)b * M + mem[q]) * D + c);
                    dot += xm * xq; nm += xm * xm; nq += xq * xq;
                }
                double cosv = (nm > 0.0 && nq > 0.0) ? dot / (sqrt(nm) * sqrt(nq)) : 0.0;
                S += cosv;
                ++npairs;
            }
            if (npairs > 0) S /= (double)npairs;
            if (window_sim_out) window_sim_out[(size_t)b * W + w] = S;
            int merge = (n >= 2) && !has_key && (S > (double)tau);
            win_merged[w] = (uint8_t)merge;
            if (merge) {
                for (int m = 0; m < n; ++m) merged_tok[mem[m]] = 1;
                rep_of[mem[0]] = w;   /* members are visited in ascending token index */
            }
        }

        /* ---- survivors in ascending original index */
        int cnt = 0;
        for (int tok = 0; tok < M; ++tok) {
            if (vb && !vb[tok]) continue;
            size_t dst = (size_t)b * M + cnt;
            if (!merged_tok[tok]) {
                memcpy((char*)out_x + dst * D * el_size(x_dtype),
                       (const char*)x + ((size_t)b * M + tok) * D * el_size(x_dtype),
                       (size_t)D * el_size(x_dtype));
                out_index[dst] = tok;
                out_mass[dst] = mb ? mb[tok] : 1.0f;
                out_is_key[dst] = is_key[tok];
                ++cnt;
            } else if (rep_of[tok] >= 0) {
                /* recover the window's members and take their mass-weighted mean */
                int w = rep_of[tok];
                int wx = w % nwx, wy = (w / nwx) % nwy, wt = w / (nwx * nwy);
                double msum = 0.0;
                for (int c = 0; c < D; ++c) mean[c] = 0.0;
                for (int dt = 0; dt < kt; ++dt)
                for (int dy = 0; dy < kh; ++dy)
                for (int dx = 0; dx < kw; ++dx) {
                    if (wt * kt + dt >= T || wy * kh + dy >= Hg || wx * kw + dx >= Wg) continue;
                    int t2 = ((wt * kt + dt) * Hg + (wy * kh + dy)) * Wg + (wx * kw + dx);
                    if (vb && !vb[t2]) continue;
                    double mm = mb ? (double)mb[t2] : 1.0;
                    msum += mm;
                    for (int c = 0; c < D; ++c)
                        mean[c] += mm * load_el(x, x_dtype, ((size_t)b * M + t2) * D + c);
                }
                for (int c = 0; c < D; ++c) store_el(out_x, x_dtype, dst * D + c, mean[c] / msum);
                out_index[dst] = tok;
                out_mass[dst] = (float)msum;
                out_is_key[dst] = 0;
                ++cnt;
            }
        }
        out_count[b] = cnt;
        if (out_valid) for (int s = 0; s < M; ++s) out_valid[(size_t)b * M + s] = (uint8_t)(s < cnt);
    }
    free(a_cls); free(logit); free(is_key); free(merged_tok); free(rep_of);
    free(order); free(mem); free(mean); free(win_merged);
    return REF_OK;
}

int mustdrop_encode_merge_ref(
    const void* x, int x_dtype,
    const void* q_cls, const void* k_cls, int qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, int key_budget,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key,
    uint8_t* out_valid, int32_t* out_count, int32_t* key_index,
    double* a_cls_out, double* window_sim_out)
{
    return encode_merge_core(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw,
                             tau, 0, key_budget, 0.0f, out_x, out_index, out_mass, out_is_key, out_valid, out_count,
                             key_index, NULL, a_cls_out, window_sim_out);
}

/* Eq. 7 as printed: O = { a_cls > mu }, mu = mean + key_lambda * std (see encode_merge_core). */
int mustdrop_encode_merge_adaptive_ref(
    const void* x, int x_dtype,
    const void* q_cls, const void* k_cls, int qk_dtype,
    const float* mass_in, const uint8_t* valid,
    int B, int T, int Hg, int Wg, int D, int Hc, int dc,
    int kt, int kh, int kw, float tau, float key_lambda, int key_cap,
    void* out_x, int32_t* out_index, float* out_mass, uint8_t* out_is_key,
    uint8_t* out_valid, int32_t* out_count, int32_t* key_index, int32_t* key_count,
    double* a_cls_out, double* window_sim_out)
{
    return encode_merge_core(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw,
                             tau, 1, key_cap, key_lambda, out_x, out_index, out_mass, out_is_key, out_valid, out_count,
                             key_index, key_count, a_cls_out, window_sim_out);
}

/* =========================================================================
 * Stage 2 -- Sec. 3.4: dual-attention filtering (Eq. 8-10) and token drop.
 * Sequence per sample: [vision 0..Mv-1 | text 0..N-1] (Sec. 3.1, prefilling).
 * ========================================================================= */
int mustdrop_prefill_filter_ref(
    const uint16_t* q_txt, const uint16_t* k, const uint16_t* v, const uint16_t* hidden,
    const uint8_t* vis_valid, const int32_t* txt_len, const uint8_t* is_key,
    int B, int Mv, int N, int H, int d, int C,
    float softmax_scale, int mode, int budget, float gamma, float alpha,
    int Rcap,
    uint16_t* hidden_out, uint16_t* k_out, uint16_t* v_out,
    int32_t* kept_index, int32_t* kept_count,
    int32_t* out_len, uint8_t* out_protect, int32_t* out_ids,
    double* score_global, double* score_indiv, double* row_lse_out)
{
    /* row_lse_out [B][H][N] (optional): the softmax normaliser of every text row as the attention of Sec. 3.4
       leaves it behind, ln sum_j exp(scale * q_i . k_j) over the keys the row sees (0 for rows >= txt_len). */
    if (B <= 0 || Mv <= 0 || N <= 0 || H <= 0 || d <= 0 || C <= 0 || Rcap <= 0) return REF_EINVAL;
    if (mode == REF_FILTER_BUDGET && (!(gamma > 0.0f) || !(alpha > 0.0f) || budget < 0)) return REF_EINVAL;
    const int L = Mv + N;
    const size_t kv_row = (size_t)H * d;
    double* a = (double*)malloc(sizeof(double) * (size_t)N * Mv);   /* head-mean probabilities, vision columns */
    double* lg = (double*)malloc(sizeof(double) * (size_t)L);
    double* Vj = (double*)malloc(sizeof(double) * (size_t)Mv);
    double* Ij = (double*)malloc(sizeof(double) * (size_t)Mv);
    uint8_t* keep = (uint8_t*)malloc((size_t)Mv);
    ranked_t* order = (ranked_t*)malloc(sizeof(ranked_t) * (size_t)Mv);

    for (int b = 0; b < B; ++b) {
        const uint8_t* vb = vis_valid ? vis_valid + (size_t)b * Mv : NULL;
        const uint8_t* kb = is_key ? is_key + (size_t)b * Mv : NULL;
        const int tl = txt_len ? txt_len[b] : N;
        if (tl < 0 || tl > N) return REF_EINVAL;

        /* a[i][j] = mean over heads of softmax_j(scale * q_i . k_j) over the keys visible to text row i */
        for (size_t t = 0; t < (size_t)N * Mv; ++t) a[t] = 0.0;
        if (row_lse_out) for (size_t t = 0; t < (size_t)H * N; ++t) row_lse_out[(size_t)b * H * N + t] = 0.0;
        for (int h = 0; h < H; ++h)
        for (int i = 0; i < tl; ++i) {
            double mx = -INFINITY;
            for (int j = 0; j < L; ++j) {
                int visible = (j < Mv) ? (!vb || vb[j]) : (j - Mv <= i);
                if (!visible) { lg[j] = -INFINITY; continue; }
                double acc = 0.0;
                for (int c = 0; c < d; ++c)
                    acc += bf16_to_double(q_txt[(((size_t)b * N + i) * H + h) * d + c]) *
                           bf16_to_double(k[(((size_t)b * L + j) * H + h) * d + c]);
                lg[j] = (double)softmax_scale * acc;
                if (lg[j] > mx) mx = lg[j];
            }
            double z = 0.0;
            for (int j = 0; j < L; ++j) if (lg[j] != -INFINITY) z += exp(lg[j] - mx);
            for (int j = 0; j < Mv; ++j)
                if (lg[j] != -INFINITY) a[(size_t)i * Mv + j] += exp(lg[j] - mx) / z / (double)H;
            if (row_lse_out) row_lse_out[((size_t)b * H + h) * N + i] = mx + log(z);
        }

        /* Eq. 8: V_j = sum_i a_ij ; Eq. 10: I_j = max_i a_ij ; Eq. 9 right side: G = sum_j V_j */
        double G = 0.0;
        int n_valid = 0;
        for (int j = 0; j < Mv; ++j) {
            double s = 0.0, m = 0.0;
            for (int i = 0; i < tl; ++i) {
                double p = a[(size_t)i * Mv + j];
                s += p;
                if (p > m) m = p;
            }
            int ok = (!vb || vb[j]);
            Vj[j] = ok ? s : 0.0;
            Ij[j] = ok ? m : 0.0;
            if (ok) { G += s; ++n_valid; }
            if (score_global) score_global[(size_t)b * Mv + j] = Vj[j];
            if (score_indiv) score_indiv[(size_t)b * Mv + j] = Ij[j];
        }

        memset(keep, 0, (size_t)Mv);
        int cnt = 0;
        if (mode == REF_FILTER_THRESHOLD) {
            /* drop j iff V_j <= gamma*G (Eq. 9) and I_j < alpha (Eq. 10) and j is not a key token */
            for (int j = 0; j < Mv; ++j) {
                if (vb && !vb[j]) continue;
                int drop = (Vj[j] <= (double)gamma * G) && (Ij[j] < (double)alpha) && !(kb && kb[j]);
                keep[j] = (uint8_t)!drop;
                cnt += !drop;
            }
        } else {
            /* budget form: the same rule with both thresholds scaled jointly until `budget` tokens pass */
            int nk = 0, no = 0;
            for (int j = 0; j < Mv; ++j) {
                if (vb && !vb[j]) continue;
                if (kb && kb[j]) { keep[j] = 1; ++nk; continue; }
                double s1 = G > 0.0 ? Vj[j] / ((double)gamma * G) : 0.0;   /* no text rows: all scores tie at 0 */
                double s2 = Ij[j] / (double)alpha;
                order[no].score = s1 > s2 ? s1 : s2;
                order[no].tie = j; order[no].slot = j; ++no;
            }
            qsort(order, (size_t)no, sizeof(ranked_t), ranked_cmp);
            int extra = budget - nk;
            if (extra < 0) extra = 0;
            if (extra > no) extra = no;
            for (int r = 0; r < extra; ++r) keep[order[r].slot] = 1;
            cnt = nk + extra;
        }
        (void)n_valid;
        kept_count[b] = cnt;   /* true count; only the first Rcap are stored */

        /* token drop: kept vision rows (ascending) then the text rows, copied bit for bit */
        int o = 0;
        for (int j = 0; j < Mv && o < Rcap; ++j) {
            if (!keep[j]) continue;
            size_t dst = (size_t)b * (Rcap + N) + o;
            size_t src = (size_t)b * L + j;
            memcpy(hidden_out + dst * C, hidden + src * C, (size_t)C * 2);
            memcpy(k_out + dst * kv_row, k + src * kv_row, kv_row * 2);
            memcpy(v_out + dst * kv_row, v + src * kv_row, kv_row * 2);
            kept_index[(size_t)b * Rcap + o] = j;
            if (out_protect) out_protect[(size_t)b * (Rcap + N) + o] = (uint8_t)(kb && kb[j]);
            if (out_ids) out_ids[(size_t)b * (Rcap + N) + o] = j;
            ++o;
        }
        for (int i = 0; i < tl; ++i) {
            size_t dst = (size_t)b * (Rcap + N) + o + i;
            size_t src = (size_t)b * L + Mv + i;
            memcpy(hidden_out + dst * C, hidden + src * C, (size_t)C * 2);
            memcpy(k_out + dst * kv_row, k + src * kv_row, kv_row * 2);
            memcpy(v_out + dst * kv_row, v + src * kv_row, kv_row * 2);
            if (out_protect) out_protect[(size_t)b * (Rcap + N) + o + i] = 1;
            if (out_ids) out_ids[(size_t)b * (Rcap + N) + o + i] = Mv + i;
        }
        if (out_ids) for (int r = o + tl; r < Rcap + N; ++r) out_ids[(size_t)b * (Rcap + N) + r] = -1;
        if (out_len) out_len[b] = o + tl;
    }
    free(a); free(lg); free(Vj); free(Ij); free(keep); free(order);
    return REF_OK;
}

/* =========================================================================
 * Stage 3 -- Sec. 3.5: output-aware cache policy, as per-step scoring of the
 * cache against the new output query (Eq. 4 attention) and eviction to a
 * budget; protected entries (the set S_few, text, generated tokens) stay.
 * ========================================================================= */
int mustdrop_decode_evict_ref(
    const uint16_t* q, uint16_t* k_cache, uint16_t* v_cache,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int B, int Lcap, int H, int d,
    float softmax_scale, float decay, int budget,
    int32_t* evicted_ids, int32_t* evicted_count,
    double* a_t_out)
{
    if (B <= 0 || Lcap <= 0 || H <= 0 || d <= 0 || budget < 0) return REF_EINVAL;
    const size_t row = (size_t)H * d;
    double* a_t = (double*)malloc(sizeof(double) * (size_t)Lcap);
    double* lg = (double*)malloc(sizeof(double) * (size_t)Lcap);
    uint8_t* keep = (uint8_t*)malloc((size_t)Lcap);
    ranked_t* order = (ranked_t*)malloc(sizeof(ranked_t) * (size_t)Lcap);

    for (int b = 0; b < B; ++b) {
        const int n = len[b];
        if (n < 0 || n > Lcap) return REF_EINVAL;
        uint16_t* kb = k_cache + (size_t)b * Lcap * row;
        uint16_t* vb = v_cache + (size_t)b * Lcap * row;
        float* ab = acc + (size_t)b * Lcap;
        int32_t* ib = ids + (size_t)b * Lcap;
        uint8_t* pb = protect + (size_t)b * Lcap;

        /* a_t[j] = mean_h softmax_j(scale * q_h . k_jh) over the live entries */
        for (int j = 0; j < n; ++j) a_t[j] = 0.0;
        for (int h = 0; h < H; ++h) {
            double mx = -INFINITY;
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int c = 0; c < d; ++c)
                    s += bf16_to_double(q[((size_t)b * H + h) * d + c]) *
                         bf16_to_double(kb[((size_t)j * H + h) * d + c]);
                lg[j] = (double)softmax_scale * s;
                if (lg[j] > mx) mx = lg[j];
            }
            double z = 0.0;
            for (int j = 0; j < n; ++j) z += exp(lg[j] - mx);
            for (int j = 0; j < n; ++j) a_t[j] += exp(lg[j] - mx) / z / (double)H;
        }
        if (a_t_out) for (int j = 0; j < Lcap; ++j) a_t_out[(size_t)b * Lcap + j] = j < n ? a_t[j] : 0.0;

        /* running score, stored in fp32 (the cache state's precision) */
        for (int j = 0; j < n; ++j) ab[j] = (float)((double)decay * (double)ab[j] + a_t[j]);

        int n_ev = 0;
        if (n > budget) {
            int np = 0, nu = 0;
            for (int j = 0; j < n; ++j) {
                if (pb[j]) { keep[j] = 1; ++np; }
                else {
                    keep[j] = 0;
                    order[nu].score = (double)ab[j]; order[nu].tie = ib[j]; order[nu].slot = j; ++nu;
                }
            }
            qsort(order, (size_t)nu, sizeof(ranked_t), ranked_cmp);
            int extra = budget - np;
            if (extra < 0) extra = 0;
            if (extra > nu) extra = nu;
            for (int r = 0; r < extra; ++r) keep[order[r].slot] = 1;
            const int new_len = np + extra;

            /* evicted ids in ascending slot order (before compaction) */
            for (int j = 0; j < n; ++j)
                if (!keep[j]) {
                    if (evicted_ids) evicted_ids[(size_t)b * Lcap + n_ev] = ib[j];
                    ++n_ev;
                }

            /* hole filling: survivors at slots >= new_len move, in ascending order,
               into the evicted slots < new_len, in ascending order */
            int hole = 0;
            for (int src = new_len; src < n; ++src) {
                if (!keep[src]) continue;
                while (keep[hole]) ++hole;
                memcpy(kb + (size_t)hole * row, kb + (size_t)src * row, row * 2);
                memcpy(vb + (size_t)hole * row, vb + (size_t)src * row, row * 2);
                ab[hole] = ab[src]; ib[hole] = ib[src]; pb[hole] = pb[src];
                keep[hole] = 1;
            }
            len[b] = new_len;
        }
        if (evicted_count) evicted_count[b] = n_ev;
    }
    free(a_t); free(lg); free(keep); free(order);
    return REF_OK;
}

/* =========================================================================
 * Stage 3, the static policy as printed (Sec. 3.5): from the shallow layers on,
 * the caches store only the vision tokens of the set S_few (and what is not a
 * vision token).  keep[b][j] != 0 marks the entries j < len[b] that stay; the
 * caches of all n_layers layers, [n_layers][B][Lcap][H][d], are compacted by
 * the hole filling of the per-step policy above, so every layer keeps the same
 * entry in the same slot.
 * ========================================================================= */
int mustdrop_decode_keep_ref(
    uint16_t* k_cache, uint16_t* v_cache, const uint8_t* keep_in,
    float* acc, int32_t* ids, uint8_t* protect, int32_t* len,
    int n_layers, int B, int Lcap, int H, int d,
    int32_t* evicted_ids, int32_t* evicted_count)
{
    if (n_layers <= 0 || B <= 0 || Lcap <= 0 || H <= 0 || d <= 0 || !keep_in) return REF_EINVAL;
    const size_t row = (size_t)H * d;
    const size_t layer = (size_t)B * Lcap * row;
    uint8_t* keep = (uint8_t*)malloc((size_t)Lcap);
    for (int b = 0; b < B; ++b) {
        const int n = len[b];
        if (n < 0 || n > Lcap) { free(keep); return REF_EINVAL; }
        float* ab = acc ? acc + (size_t)b * Lcap : NULL;
        int32_t* ib = ids + (size_t)b * Lcap;
        uint8_t* pb = protect + (size_t)b * Lcap;
        int new_len = 0, n_ev = 0;
        for (int j = 0; j < n; ++j) {
            keep[j] = keep_in[(size_t)b * Lcap + j] != 0;
            new_len += keep[j];
        }
        for (int j = 0; j < n; ++j)
            if (!keep[j]) {
                if (evicted_ids) evicted_ids[(size_t)b * Lcap + n_ev] = ib[j];
                ++n_ev;
            }
        int hole = 0;
        for (int src = new_len; src < n; ++src) {
            if (!keep[src]) continue;
            while (keep[hole]) ++hole;
            for (int l = 0; l < n_layers; ++l) {
                uint16_t* kb = k_cache + l * layer + (size_t)b * Lcap * row;
                uint16_t* vb = v_cache + l * layer + (size_t)b * Lcap * row;
                memcpy(kb + (size_t)hole * row, kb + (size_t)src * row, row * 2);
                memcpy(vb + (size_t)hole * row, vb + (size_t)src * row, row * 2);
            }
            if (ab) ab[hole] = ab[src];
            ib[hole] = ib[src]; pb[hole] = pb[src];
            keep[hole] = 1;
        }
        len[b] = new_len;
        if (evicted_count) evicted_count[b] = n_ev;
    }
    free(keep);
    return REF_OK;
}
