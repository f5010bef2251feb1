/* Sanitizer driver of the CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Built together with mustdrop_ref.c under -fsanitize=address,undefined and run by a CPU test:
 * every oracle entry point on small seeded inputs that exercise the ragged cases (clipped border
 * windows, padded vision slots, short prompts, more keys than budget, empty caches), with every
 * buffer allocated at its exact size so that an access one element too far is a report.
 * It checks nothing about the values (the pins do that); it only has to run clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int mustdrop_encode_merge_ref(const void*, int, const void*, const void*, int, const float*, const uint8_t*,
                              int, int, int, int, int, int, int, int, int, int, float, int,
                              void*, int32_t*, float*, uint8_t*, uint8_t*, int32_t*, int32_t*, double*, double*);
int mustdrop_encode_merge_adaptive_ref(const void*, int, const void*, const void*, int, const float*, const uint8_t*,
                                       int, int, int, int, int, int, int, int, int, int, float, float, int,
                                       void*, int32_t*, float*, uint8_t*, uint8_t*, int32_t*, int32_t*, int32_t*, double*, double*);
int mustdrop_prefill_filter_ref(const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                const uint8_t*, const int32_t*, const uint8_t*, int, int, int, int, int, int,
                                float, int, int, float, float, int,
                                uint16_t*, uint16_t*, uint16_t*, int32_t*, int32_t*, int32_t*, uint8_t*, int32_t*,
                                double*, double*, double*);
int mustdrop_decode_evict_ref(const uint16_t*, uint16_t*, uint16_t*, float*, int32_t*, uint8_t*, int32_t*,
                              int, int, int, int, float, float, int, int32_t*, int32_t*, double*);
int mustdrop_decode_keep_ref(uint16_t*, uint16_t*, const uint8_t*, float*, int32_t*, uint8_t*, int32_t*,
                             int, int, int, int, int, int32_t*, int32_t*);

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double uniform(void) {                       /* splitmix64 -> [0, 1) */
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (double)(z >> 11) / 9007199254740992.0;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(uniform() + 1e-300)) * cos(6.283185307179586 * uniform())); }
static uint16_t bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16); }
static void* xmalloc(size_t n) { void* p = malloc(n ? n : 1); if (!p) { fprintf(stderr, "out of memory\n"); exit(2); } return p; }
static uint16_t* rand_bf16(size_t n) { uint16_t* p = xmalloc(2 * n); for (size_t i = 0; i < n; ++i) p[i] = bf16(gauss()); return p; }
static float* rand_f32(size_t n) { float* p = xmalloc(4 * n); for (size_t i = 0; i < n; ++i) p[i] = gauss(); return p; }
static uint8_t* rand_mask(size_t n, double p_one) { uint8_t* p = xmalloc(n); for (size_t i = 0; i < n; ++i) p[i] = uniform() < p_one; return p; }
#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s:%d: rc=%d\n", __FILE__, __LINE__, rc_); return 1; } } while (0)

static int run_encode(int dtype, int B, int T, int Hg, int Wg, int D, int Hc, int kt, int kh, int kw, int key_budget,
                      int with_mask, int with_mass, int adaptive) {
    const int M = T * Hg * Wg, dc = D / Hc;
    const int W = ((T + kt - 1) / kt) * ((Hg + kh - 1) / kh) * ((Wg + kw - 1) / kw);
    void* x = dtype ? (void*)rand_bf16((size_t)B * M * D) : (void*)rand_f32((size_t)B * M * D);
    void* q = dtype ? (void*)rand_bf16((size_t)B * D) : (void*)rand_f32((size_t)B * D);
    void* k = dtype ? (void*)rand_bf16((size_t)B * (M + 1) * D) : (void*)rand_f32((size_t)B * (M + 1) * D);
    uint8_t* valid = with_mask ? rand_mask((size_t)B * M, 0.7) : NULL;
    float* mass = NULL;
    if (with_mass) { mass = xmalloc(4 * (size_t)B * M); for (int i = 0; i < B * M; ++i) mass[i] = 1.0f + (float)(int)(3 * uniform()); }
    void* out_x = xmalloc((size_t)B * M * D * (dtype ? 2 : 4));
    int32_t* out_index = xmalloc(4 * (size_t)B * M);
    float* out_mass = xmalloc(4 * (size_t)B * M);
    uint8_t* out_is_key = xmalloc((size_t)B * M);
    uint8_t* out_valid = xmalloc((size_t)B * M);
    int32_t* out_count = xmalloc(4 * (size_t)B);
    const int cap = adaptive ? M : key_budget;
    int32_t* key_index = xmalloc(4 * (size_t)B * (cap > 0 ? cap : 1));
    int32_t* key_count = xmalloc(4 * (size_t)B);
    double* a_cls = xmalloc(8 * (size_t)B * M);
    double* wsim = xmalloc(8 * (size_t)B * W);
    if (adaptive)
        CHECK(mustdrop_encode_merge_adaptive_ref(x, dtype, q, k, dtype, mass, valid, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, 0.2f, 1.0f,
                                                 cap, out_x, out_index, out_mass, out_is_key, out_valid, out_count, key_index,
                                                 key_count, a_cls, wsim));
    else
        CHECK(mustdrop_encode_merge_ref(x, dtype, key_budget ? q : NULL, key_budget ? k : NULL, dtype, mass, valid, B, T, Hg, Wg, D,
                                        key_budget ? Hc : 1, key_budget ? dc : D, kt, kh, kw, 0.0f, key_budget, out_x, out_index,
                                        out_mass, out_is_key, out_valid, out_count, key_index, a_cls, wsim));
    free(x); free(q); free(k); free(valid); free(mass); free(out_x); free(out_index); free(out_mass); free(out_is_key);
    free(out_valid); free(out_count); free(key_index); free(key_count); free(a_cls); free(wsim);
    return 0;
}

static int run_prefill(int B, int Mv, int N, int H, int d, int C, int mode, int budget, int Rcap, int masks) {
    const size_t L = (size_t)Mv + N;
    uint16_t* q = rand_bf16((size_t)B * N * H * d);
    uint16_t* k = rand_bf16(B * L * H * d);
    uint16_t* v = rand_bf16(B * L * H * d);
    uint16_t* hid = rand_bf16(B * L * C);
    uint8_t* vv = masks ? rand_mask((size_t)B * Mv, 0.6) : NULL;
    uint8_t* key = masks ? rand_mask((size_t)B * Mv, 0.1) : NULL;
    int32_t* tl = NULL;
    if (masks) { tl = xmalloc(4 * (size_t)B); for (int b = 0; b < B; ++b) tl[b] = b == 0 ? N : 1 + (int)(uniform() * (N - 1)); }
    const size_t rows = (size_t)Rcap + N;
    uint16_t* ho = xmalloc(2 * B * rows * C);
    uint16_t* ko = xmalloc(2 * B * rows * H * d);
    uint16_t* vo = xmalloc(2 * B * rows * H * d);
    int32_t* kept = xmalloc(4 * (size_t)B * Rcap);
    int32_t* cnt = xmalloc(4 * (size_t)B);
    int32_t* olen = xmalloc(4 * (size_t)B);
    uint8_t* prot = xmalloc(B * rows);
    int32_t* ids = xmalloc(4 * B * rows);
    double* sg = xmalloc(8 * (size_t)B * Mv);
    double* si = xmalloc(8 * (size_t)B * Mv);
    double* lse = xmalloc(8 * (size_t)B * H * N);
    CHECK(mustdrop_prefill_filter_ref(q, k, v, hid, vv, tl, key, B, Mv, N, H, d, C, 1.0f / sqrtf((float)d), mode, budget,
                                      1.0f / Mv, 2.0f / (Mv + N), Rcap, ho, ko, vo, kept, cnt, olen, prot, ids, sg, si, lse));
    free(q); free(k); free(v); free(hid); free(vv); free(key); free(tl); free(ho); free(ko); free(vo); free(kept); free(cnt);
    free(olen); free(prot); free(ids); free(sg); free(si); free(lse);
    return 0;
}

static int run_decode(int B, int Lcap, int H, int d, int budget, int layers) {
    uint16_t* q = rand_bf16((size_t)B * H * d);
    uint16_t* kc = rand_bf16((size_t)layers * B * Lcap * H * d);
    uint16_t* vc = rand_bf16((size_t)layers * B * Lcap * H * d);
    float* acc = xmalloc(4 * (size_t)B * Lcap);
    int32_t* ids = xmalloc(4 * (size_t)B * Lcap);
    uint8_t* prot = rand_mask((size_t)B * Lcap, 0.15);
    uint8_t* keep = rand_mask((size_t)B * Lcap, 0.5);
    int32_t* len = xmalloc(4 * (size_t)B);
    int32_t* ev = xmalloc(4 * (size_t)B * Lcap);
    int32_t* evc = xmalloc(4 * (size_t)B);
    double* at = xmalloc(8 * (size_t)B * Lcap);
    for (int i = 0; i < B * Lcap; ++i) { acc[i] = (float)uniform(); ids[i] = i % Lcap; }
    for (int b = 0; b < B; ++b) len[b] = b == 0 ? Lcap : (b == 1 ? 0 : 1 + (int)(uniform() * (Lcap - 1)));
    CHECK(mustdrop_decode_evict_ref(q, kc, vc, acc, ids, prot, len, B, Lcap, H, d, 1.0f / sqrtf((float)d), 0.5f, budget, ev, evc, at));
    for (int b = 0; b < B; ++b) len[b] = b == 0 ? Lcap : (b == 1 ? 0 : len[b]);
    CHECK(mustdrop_decode_keep_ref(kc, vc, keep, acc, ids, prot, len, layers, B, Lcap, H, d, ev, evc));
    free(q); free(kc); free(vc); free(acc); free(ids); free(prot); free(keep); free(len); free(ev); free(evc); free(at);
    return 0;
}

int main(void) {
    /* stage 1: fp32 and bf16, windows that divide the grid and windows clipped at the border, video windows */
    if (run_encode(0, 2, 1, 6, 6, 32, 4, 1, 2, 2, 5, 0, 0, 0)) return 1;
    if (run_encode(1, 3, 1, 7, 5, 64, 4, 1, 2, 2, 9, 1, 1, 0)) return 1;
    if (run_encode(1, 2, 3, 4, 6, 32, 2, 2, 2, 2, 0, 1, 0, 0)) return 1;
    if (run_encode(1, 2, 2, 5, 5, 32, 2, 2, 3, 3, 4, 1, 1, 1)) return 1;
    /* stage 2: both modes, masks and short prompts, more keys than budget, capacity below the kept count */
    if (run_prefill(2, 37, 9, 3, 16, 24, 0, 12, 12, 0)) return 1;
    if (run_prefill(3, 50, 17, 2, 32, 16, 0, 3, 3, 1)) return 1;
    if (run_prefill(2, 33, 5, 2, 16, 8, 1, 0, 33, 1)) return 1;
    if (run_prefill(2, 33, 5, 2, 16, 8, 1, 0, 4, 1)) return 1;
    /* stage 3: full, empty and partly filled caches; budgets above and below the live length */
    if (run_decode(4, 40, 3, 16, 12, 2)) return 1;
    if (run_decode(3, 17, 2, 8, 64, 1)) return 1;
    if (run_decode(3, 9, 1, 8, 0, 3)) return 1;
    printf("oracle sanitize: ok\n");
    return 0;
}
