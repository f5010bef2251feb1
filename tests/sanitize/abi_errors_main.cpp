// Sanitizer driver of the C ABI's host side: the library is built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the HOST pass only and this program walks the argument checks of every
// entry point -- calls that must be rejected before any kernel is launched, with pointers that are never
// dereferenced on the host -- and the workspace-size arithmetic at small, odd and very large shapes.  No
// GPU is needed: every call returns from the host-side checks.  It has to run clean and see the codes it
// expects.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/mustdrop.h"
#include "../../include/mustdrop_bench.h"

static int g_fail = 0;
#define EXPECT(call, code)                                                                              \
    do {                                                                                                \
        const int rc_ = (call);                                                                         \
        if (rc_ != (code)) { std::fprintf(stderr, "%s:%d: got %d (%s), expected %d\n", __FILE__, __LINE__, rc_, mustdrop_last_error(), (int)(code)); ++g_fail; } \
        else if ((code) != MD_OK && std::strlen(mustdrop_last_error()) == 0) { std::fprintf(stderr, "%s:%d: no message\n", __FILE__, __LINE__); ++g_fail; } \
    } while (0)

// distinct, aligned addresses far apart (never dereferenced by the host code under test)
static void* fake(int i) { return reinterpret_cast<void*>((uintptr_t)0x100000000ull + (uintptr_t)i * 0x40000000ull); }

int main() {
    void *X = fake(1), *Q = fake(2), *K = fake(3), *OX = fake(4), *WS = fake(5);
    int32_t *OI = (int32_t*)fake(6), *OC = (int32_t*)fake(7), *KI = (int32_t*)fake(8), *KC = (int32_t*)fake(9);
    float* OM = (float*)fake(10);
    uint8_t *OK_ = (uint8_t*)fake(11), *OV = (uint8_t*)fake(12);
    const size_t big = (size_t)1 << 40;

    if (mustdrop_version() < 1) { std::fprintf(stderr, "version\n"); return 1; }
    // ---- workspace arithmetic: monotone, aligned, zero for bad shapes, no overflow at the limits
    size_t a = mustdrop_encode_merge_workspace_bytes(16, 1, 24, 24, 16, 1, 2, 2), b = mustdrop_encode_merge_workspace_bytes(32, 1, 24, 24, 16, 1, 2, 2);
    if (!(a > 0 && a < b && a % 256 == 0)) { std::fprintf(stderr, "encode workspace %zu %zu\n", a, b); ++g_fail; }
    if (mustdrop_encode_merge_workspace_bytes(0, 1, 24, 24, 16, 1, 2, 2) != 0) ++g_fail;
    (void)mustdrop_encode_merge_workspace_bytes(64, 8, 64, 64, 256, 2, 2, 2);
    (void)mustdrop_encode_merge_workspace_bytes(1, 1, 27, 27, 16, 1, 2, 2);
    for (int N : {1, 31, 32, 33, 128, 300, 4096})
        for (int Mv : {1, 127, 576, 2880, 65536})
            if (mustdrop_prefill_filter_workspace_bytes(3, Mv, N, 32, Mv < 64 ? Mv : 64) == 0) { std::fprintf(stderr, "prefill workspace %d %d\n", Mv, N); ++g_fail; }
    if (mustdrop_prefill_filter_workspace_bytes(0, 576, 64, 32, 192) != 0) ++g_fail;
    (void)mustdrop_prefill_filter_workspace_bytes(4096, 65536, 4096, 128, 65536);
    if (mustdrop_decode_evict_workspace_bytes(64, 4352, 32) == 0 || mustdrop_decode_evict_workspace_bytes(0, 10, 1) != 0) ++g_fail;
    (void)mustdrop_decode_evict_workspace_bytes(4096, 1 << 20, 1024);

    // ---- stage 1
#define ENC(x, xd, q, k, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, tau, kb, ox, ws, wsb)                       \
    mustdrop_encode_merge(x, xd, q, k, MD_BF16, nullptr, nullptr, B, T, Hg, Wg, D, Hc, dc, kt, kh, kw, tau, kb, ox, OI, OM, OK_, OV, OC, KI, nullptr, nullptr, ws, wsb, nullptr)
    EXPECT(ENC(nullptr, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EINVAL);
    EXPECT(ENC(X, (md_dtype)7, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EDTYPE);
    EXPECT(ENC(X, MD_BF16, Q, K, 0, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EINVAL);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 3, 3, 3, 0.9f, 4, OX, WS, big), MD_ESHAPE);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 8, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_ESHAPE);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 60, 4, 15, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EALIGN);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 65, OX, WS, big), MD_EINVAL);
    EXPECT(ENC(X, MD_BF16, nullptr, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EINVAL);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, X, WS, big), MD_EALIAS);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, 16), MD_EWORKSPACE);
    EXPECT(ENC(X, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, (char*)WS + 8, big), MD_EALIGN);
    EXPECT(ENC((char*)X + 2, MD_BF16, Q, K, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 4, OX, WS, big), MD_EALIGN);
    EXPECT(mustdrop_encode_merge_adaptive(X, MD_BF16, Q, K, MD_BF16, nullptr, nullptr, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 1.0f, 8, OX, OI, OM,
                                          OK_, OV, OC, KI, nullptr, nullptr, nullptr, WS, big, nullptr), MD_EINVAL);      // key_count missing
    EXPECT(mustdrop_encode_merge_adaptive(X, MD_BF16, Q, K, MD_BF16, nullptr, nullptr, 2, 1, 8, 8, 64, 4, 16, 1, 2, 2, 0.9f, 0.0f / 0.0f * 0 + __builtin_nanf(""), 8,
                                          OX, OI, OM, OK_, OV, OC, KI, KC, nullptr, nullptr, WS, big, nullptr), MD_EINVAL);
    EXPECT(mustdrop_encode_merge_noalloc(X, MD_BF16, Q, K, MD_BF16, nullptr, nullptr, 200, 8, 24, 24, 1024, 16, 64, 2, 2, 2, 0.9f, 32, OX, OI, OM, OK_,
                                         OV, OC, KI, nullptr, nullptr, nullptr), MD_EWORKSPACE);

    // ---- stage 2
    void *QT = fake(13), *KK = fake(14), *VV = fake(15), *HH = fake(16), *HO = fake(17), *KO = fake(18), *VO = fake(19);
    int32_t *KEPT = (int32_t*)fake(20), *KCNT = (int32_t*)fake(21), *OLEN = (int32_t*)fake(22), *OIDS = (int32_t*)fake(23);
    uint8_t* OPROT = (uint8_t*)fake(24);
#define PRE(q, B, Mv, N, H, d, C, mode, budget, gamma, alpha, Rcap, ho, ws, wsb)                           \
    mustdrop_prefill_filter(q, KK, VV, HH, nullptr, nullptr, nullptr, nullptr, B, Mv, N, H, d, C, 0.088f, mode, budget, gamma, alpha, Rcap, ho, KO, VO, \
                            KEPT, KCNT, OLEN, OPROT, OIDS, nullptr, nullptr, ws, wsb, nullptr)
    EXPECT(PRE(nullptr, 2, 64, 16, 4, 128, 256, MD_FILTER_BUDGET, 8, 0.01f, 0.02f, 8, HO, WS, big), MD_EINVAL);
    EXPECT(PRE(QT, 2, 0, 16, 4, 128, 256, MD_FILTER_BUDGET, 8, 0.01f, 0.02f, 8, HO, WS, big), MD_EINVAL);
    EXPECT(PRE(QT, 2, 64, 16, 4, 96, 256, MD_FILTER_BUDGET, 8, 0.01f, 0.02f, 8, HO, WS, big), MD_ESHAPE);
    EXPECT(PRE(QT, 2, 64, 16, 4, 128, 256, (md_filter_mode)9, 8, 0.01f, 0.02f, 8, HO, WS, big), MD_EDTYPE);
    EXPECT(PRE(QT, 2, 64, 16, 4, 128, 256, MD_FILTER_BUDGET, 8, -1.0f, 0.02f, 8, HO, WS, big), MD_EINVAL);
    EXPECT(PRE(QT, 2, 64, 16, 4, 128, 256, MD_FILTER_BUDGET, 8, 0.01f, 0.02f, 8, HH, WS, big), MD_EALIAS);
    EXPECT(PRE(QT, 2, 64, 16, 4, 128, 256, MD_FILTER_BUDGET, 8, 0.01f, 0.02f, 8, HO, WS, 64), MD_EWORKSPACE);
    md_kv_layout lq{16 * 4 * 128, 4 * 128, 128}, lkv{80 * 4 * 128, 4 * 128, 128}, lo{24 * 4 * 128, 4 * 128, 128}, bad{80 * 4 * 128, 4 * 128, 100};
    EXPECT(mustdrop_prefill_filter_strided(QT, KK, VV, HH, nullptr, nullptr, nullptr, nullptr, 2, 64, 16, 4, 128, 256, 0.088f, MD_FILTER_BUDGET, 8, 0.01f,
                                           0.02f, 8, HO, KO, VO, KEPT, KCNT, OLEN, OPROT, OIDS, nullptr, nullptr, &lq, &bad, &lo, WS, big, nullptr), MD_EINVAL);
    (void)lkv;

    // ---- stage 3
    void *DQ = fake(25), *KCA = fake(26), *VCA = fake(27);
    float* ACC = (float*)fake(28);
    int32_t *IDS = (int32_t*)fake(29), *LEN = (int32_t*)fake(30);
    uint8_t *PROT = (uint8_t*)fake(31), *KEEP = (uint8_t*)fake(32);
#define DEC(q, acc, B, Lcap, H, d, decay, budget, ws, wsb)                                                \
    mustdrop_decode_evict(q, KCA, VCA, acc, IDS, PROT, LEN, B, Lcap, H, d, 0.088f, decay, budget, nullptr, nullptr, ws, wsb, nullptr)
    EXPECT(DEC(nullptr, ACC, 2, 64, 4, 128, 1.0f, 16, WS, big), MD_EINVAL);
    EXPECT(DEC(DQ, ACC, 2, 64, 4, 100, 1.0f, 16, WS, big), MD_ESHAPE);
    EXPECT(DEC(DQ, ACC, 2, 64, 4, 128, -0.5f, 16, WS, big), MD_EINVAL);
    EXPECT(DEC(DQ, ACC, 2, 64, 4, 128, 1.0f, -1, WS, big), MD_EINVAL);
    EXPECT(DEC(DQ, (float*)IDS, 2, 64, 4, 128, 1.0f, 16, WS, big), MD_EALIAS);
    EXPECT(DEC(DQ, ACC, 2, 64, 4, 128, 1.0f, 16, WS, 8), MD_EWORKSPACE);
    EXPECT(mustdrop_decode_append(nullptr, VCA, KCA, VCA, ACC, IDS, PROT, LEN, 2, 64, 4, 128, 7, 1, nullptr), MD_EINVAL);
    EXPECT(mustdrop_decode_keep(KCA, VCA, nullptr, ACC, IDS, PROT, LEN, 2, 2, 64, 4, 128, nullptr, nullptr, WS, big, nullptr), MD_EINVAL);
    EXPECT(mustdrop_decode_keep(KCA, VCA, KEEP, ACC, IDS, PROT, LEN, 0, 2, 64, 4, 128, nullptr, nullptr, WS, big, nullptr), MD_EINVAL);
    md_kv_layout cl{64 * 4 * 128, 4 * 128, 128};
    EXPECT(mustdrop_decode_keep_strided(KCA, VCA, KEEP, ACC, IDS, PROT, LEN, 3, 2, 64, 4, 128, nullptr, nullptr, &cl, 12, WS, big, nullptr), MD_ESHAPE);
    EXPECT(mustdrop_decode_evict_strided(DQ, KCA, VCA, ACC, IDS, PROT, LEN, 2, 64, 4, 128, 0.088f, 1.0f, 16, nullptr, nullptr, &bad, WS, big, nullptr), MD_EINVAL);

    // ---- the benchmarking aid with nothing recorded
    EXPECT(mustdrop_profile_stop(nullptr, nullptr, nullptr, 0, nullptr), MD_OK);

    if (g_fail) { std::fprintf(stderr, "abi sanitize: %d unexpected result(s)\n", g_fail); return 1; }
    std::printf("abi sanitize: ok\n");
    return 0;
}
