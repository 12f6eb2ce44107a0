// Host-only driver for the AddressSanitizer / UndefinedBehaviorSanitizer build (tests/test_host_sanitizers.py):
// runs the CPU oracle and the library's host code -- layout builder, introspection, cache geometry, argument checks
// of the entry points (HIP stubbed out: hip_stub/) -- over a spread of shapes, and cross-checks the library's mask and
// tile schedule against the oracle's predicate on the way.  Exit status 0 = all checks passed; the sanitizers abort
// the run on any finding.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ksa.h"
#include "ksa_internal.h"

extern "C" {
int64_t ksa_oracle_aug_len(int64_t n, int32_t c, int32_t m);
int ksa_oracle_visible(int64_t aq, int64_t ak, int32_t c, int32_t m, int32_t C, uint32_t flags);
void ksa_oracle_mask_row(int64_t aq, int64_t L, int32_t c, int32_t m, int32_t C, uint32_t flags, uint8_t *row);
int ksa_oracle_index_maps(int64_t n, int32_t c, int32_t m, int32_t *aug_chunk, uint8_t *aug_is_summary,
                          int32_t *position_ids, int32_t *text_to_aug, int32_t *summary_to_aug);
int ksa_oracle_prefill(const float *q, const float *k, const float *v, int32_t B, int64_t n, int32_t c, int32_t m,
                       int32_t C, int32_t Hq, int32_t Hkv, int32_t d, double scale, uint32_t flags,
                       const int64_t *rows, int64_t n_rows, double *o, double *lse);
int ksa_oracle_row_weights(const float *q, const float *k, int32_t B, int64_t n, int32_t c, int32_t m, int32_t C,
                           int32_t Hq, int32_t Hkv, int32_t d, double scale, uint32_t flags, int32_t b, int32_t h,
                           int64_t aq, double *weight_out, double *lse_out);
int ksa_oracle_prefill_bwd(const float *q, const float *k, const float *v, const float *g, int32_t B, int64_t n,
                           int32_t c, int32_t m, int32_t C, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                           uint32_t flags, const int64_t *q_rows, int64_t n_q_rows, const int64_t *k_rows,
                           int64_t n_k_rows, double *dq, double *dk, double *dv);
int ksa_oracle_decode(const float *q, const float *k_sum, const float *v_sum, int64_t S, const float *k_txt,
                      const float *v_txt, int64_t W, const int64_t *txt_base, const int64_t *pos, int32_t B, int32_t c,
                      int32_t m, int32_t C, int32_t Hq, int32_t Hkv, int32_t d, double scale, double *o, double *lse);
}

// The launchers live in the .hip files; in this build nothing may reach them.
size_t ksa_prefill_workspace_size(const ksa_params &p) {
    const int64_t n_sum = (int64_t)(p.n_text / p.chunk_len) * p.n_summary;
    return (size_t)((int64_t)p.batch * p.n_kv_heads * p.head_dim * ((p.n_text + 63) / 64 * 64 + (n_sum + 63) / 64 * 64) * 2);
}
size_t ksa_prefill_bwd_workspace_size(const ksa_params &, int64_t aug_len) { return (size_t)aug_len * 8; }
int ksa_launch_prefill(const KsaPrefillLaunch &, void *) { return KSA_ERR_HIP; }
int ksa_launch_prefill_bwd(const KsaPrefillBwdLaunch &, void *) { return KSA_ERR_HIP; }
int ksa_launch_decode(const KsaDecodeLaunch &, void *) { return KSA_ERR_HIP; }
int ksa_launch_cache_fill(const KsaCacheFillLaunch &, void *) { return KSA_ERR_HIP; }
int ksa_launch_cache_append(const KsaCacheAppendLaunch &, void *) { return KSA_ERR_HIP; }
int ksa_decode_default_splits(const ksa_params *) { return 2; }
int ksa_decode_static_scratch(float **) { return KSA_ERR_HIP; }

static int failures = 0;
#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond);       \
            ++failures;                                                          \
        }                                                                        \
    } while (0)

static ksa_params make(int B, int n, int c, int m, int C, int Hq, int Hkv, int d, unsigned flags) {
    ksa_params p;
    std::memset(&p, 0, sizeof(p));
    p.batch = B, p.n_text = n, p.chunk_len = c, p.n_summary = m, p.compress_ratio = m ? c / m : 0, p.window_chunks = C;
    p.n_q_heads = Hq, p.n_kv_heads = Hkv, p.head_dim = d, p.softmax_scale = 0.f, p.flags = flags;
    return p;
}

static unsigned rng_state = 12345u;
static float rnd() {
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}

static void layout_against_oracle(int n, int c, int m, int C, unsigned flags, int Hq, int Hkv) {
    ksa_params p = make(1, n, c, m, C, Hq, Hkv, 128, flags);
    ksa_layout *lay = nullptr;
    CHECK(ksa_build_layout(&p, &lay) == KSA_OK && lay);
    if (!lay) return;
    int64_t L = 0;
    int32_t J = 0, qt = 0, kt = 0, hs = 0;
    CHECK(ksa_layout_dims(lay, &L, &J, &qt, &kt, &hs) == KSA_OK);
    CHECK(L == ksa_oracle_aug_len(n, c, m));
    int64_t rows_fn = -1;
    CHECK(ksa_augmented_rows(&p, n, &rows_fn) == KSA_OK && rows_fn == L);
    // index maps
    std::vector<int32_t> a1(L), p1(L), t1(n), s1((size_t)J * m + 1), a2(L), p2(L), t2(n), s2((size_t)J * m + 1);
    std::vector<uint8_t> i1(L), i2(L);
    CHECK(ksa_layout_index_maps(lay, a1.data(), i1.data(), p1.data(), t1.data(), s1.data()) == KSA_OK);
    CHECK(ksa_oracle_index_maps(n, c, m, a2.data(), i2.data(), p2.data(), t2.data(), s2.data()) == 0);
    CHECK(a1 == a2 && i1 == i2 && p1 == p2 && t1 == t2);
    for (int x = 0; x < J * m; ++x) CHECK(s1[x] == s2[x]);
    // mask rows
    std::vector<uint8_t> r1(L), r2(L);
    std::vector<std::vector<int>> cover(L, std::vector<int>(L, 0));
    for (int64_t a = 0; a < L; ++a) {
        CHECK(ksa_layout_mask_row(lay, a, r1.data()) == KSA_OK);
        ksa_oracle_mask_row(a, L, c, m, C, flags, r2.data());
        CHECK(r1 == r2);
        int32_t rg[4];
        CHECK(ksa_layout_row_ranges(lay, a, rg) == KSA_OK);
    }
    CHECK(ksa_layout_mask_row(lay, L, r1.data()) == KSA_ERR_OUT_OF_RANGE);
    // tile schedule: every visible pair in exactly one visited tile
    int64_t np = 0;
    CHECK(ksa_layout_tile_pairs(lay, &np, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == KSA_OK);
    std::vector<uint8_t> qs(np), ks(np), kind(np);
    std::vector<int32_t> qb(np), qc(np), kb(np), kc(np);
    CHECK(ksa_layout_tile_pairs(lay, &np, qs.data(), qb.data(), qc.data(), ks.data(), kb.data(), kc.data(), kind.data()) == KSA_OK);
    for (int64_t x = 0; x < np; ++x)
        for (int qi = qb[x]; qi < qb[x] + qc[x]; ++qi) {
            const int64_t aq = qs[x] == KSA_SPACE_TEXT ? t1[qi] : s1[qi];
            int32_t rg[4];
            ksa_layout_row_ranges(lay, aq, rg);
            const int lo = ks[x] == KSA_SPACE_TEXT ? rg[2] : rg[0], hi = ks[x] == KSA_SPACE_TEXT ? rg[3] : rg[1];
            for (int ki = kb[x]; ki < kb[x] + kc[x]; ++ki) {
                const bool vis = ki >= lo && ki < hi;
                if (kind[x] == KSA_TILE_FULL) CHECK(vis);
                if (vis) cover[aq][ks[x] == KSA_SPACE_TEXT ? t1[ki] : s1[ki]] += 1;
            }
        }
    for (int64_t a = 0; a < L; ++a)
        for (int64_t b = 0; b < L; ++b) CHECK(cover[a][b] == ksa_oracle_visible(a, b, c, m, C, flags));
    int64_t ne = 0;
    CHECK(ksa_layout_launch_order(lay, &ne, nullptr, nullptr, nullptr, nullptr) == KSA_OK && ne % 8 == 0);
    std::vector<uint8_t> es(ne);
    std::vector<int32_t> eb(ne), ebat(ne), eh(ne);
    CHECK(ksa_layout_launch_order(lay, &ne, es.data(), eb.data(), ebat.data(), eh.data()) == KSA_OK);
    CHECK(ksa_prefill_workspace_bytes(lay) > 0);
    // entry points: everything in front of the first HIP call
    int dummy[64] = {0};
    CHECK(ksa_prefill_fwd(lay, nullptr, dummy, dummy, dummy, nullptr, nullptr, nullptr, nullptr, dummy, 1 << 30, nullptr) == KSA_ERR_INVALID_ARG);
    CHECK(ksa_prefill_fwd(lay, dummy, dummy, dummy, dummy, nullptr, nullptr, nullptr, nullptr, dummy, 16, nullptr) == KSA_ERR_WORKSPACE_TOO_SMALL);
    const int64_t bad[3] = {8, 7, 8};
    CHECK(ksa_prefill_fwd(lay, dummy, dummy, dummy, dummy, nullptr, bad, nullptr, nullptr, dummy, (size_t)1 << 40, nullptr) == KSA_ERR_INVALID_ARG);
    CHECK(ksa_prefill_fwd(lay, dummy, dummy, dummy, dummy, nullptr, nullptr, nullptr, nullptr, dummy, (size_t)1 << 40, nullptr) == KSA_ERR_HIP);
    CHECK(ksa_layout_upload(lay) == KSA_ERR_HIP);
    ksa_layout_destroy(lay);
}

static void oracle_numerics(int n, int c, int m, int C, unsigned flags) {
    const int B = 2, Hq = 4, Hkv = 2, d = 8;
    const int64_t L = ksa_oracle_aug_len(n, c, m);
    std::vector<float> q((size_t)B * L * Hq * d), k((size_t)B * L * Hkv * d), v(k.size()), g(q.size());
    for (auto &x : q) x = rnd();
    for (auto &x : k) x = rnd();
    for (auto &x : v) x = 1.0f;
    for (auto &x : g) x = rnd();
    std::vector<double> o((size_t)B * L * Hq * d), lse((size_t)B * Hq * L);
    CHECK(ksa_oracle_prefill(q.data(), k.data(), v.data(), B, n, c, m, C, Hq, Hkv, d, 0.0, flags, nullptr, 0, o.data(), lse.data()) == 0);
    for (double x : o) CHECK(x > 1.0 - 1e-12 && x < 1.0 + 1e-12);   // V == 1 gives O == 1: weights sum to one
    const int64_t rows[3] = {0, L / 2, L - 1};
    std::vector<double> o3((size_t)B * 3 * Hq * d), l3((size_t)B * Hq * 3);
    CHECK(ksa_oracle_prefill(q.data(), k.data(), v.data(), B, n, c, m, C, Hq, Hkv, d, 0.3, flags, rows, 3, o3.data(), l3.data()) == 0);
    std::vector<double> w(L);
    double l = 0;
    CHECK(ksa_oracle_row_weights(q.data(), k.data(), B, n, c, m, C, Hq, Hkv, d, 0.0, flags, 1, 3, L - 1, w.data(), &l) == 0);
    double sum = 0;
    for (double x : w) sum += x;
    CHECK(sum > 1.0 - 1e-12 && sum < 1.0 + 1e-12);
    for (auto &x : v) x = rnd();
    std::vector<double> dq(o.size()), dk((size_t)B * L * Hkv * d), dv(dk.size());
    CHECK(ksa_oracle_prefill_bwd(q.data(), k.data(), v.data(), g.data(), B, n, c, m, C, Hq, Hkv, d, 0.0, flags, nullptr, 0, nullptr, 0, dq.data(), dk.data(), dv.data()) == 0);
    const int64_t some[2] = {1, L - 1};
    std::vector<double> dq2((size_t)B * 2 * Hq * d), dk2((size_t)B * 2 * Hkv * d), dv2(dk2.size());
    CHECK(ksa_oracle_prefill_bwd(q.data(), k.data(), v.data(), g.data(), B, n, c, m, C, Hq, Hkv, d, 0.0, flags, some, 2, some, 2, dq2.data(), dk2.data(), dv2.data()) == 0);
    CHECK(ksa_oracle_prefill(q.data(), k.data(), v.data(), B, n, c, m, C, 3, 2, d, 0.0, flags, nullptr, 0, o.data(), lse.data()) == -1);
}

static void decode_checks(int n_cap, int c, int m, int C) {
    ksa_params p = make(2, n_cap, c, m, C, 4, 2, 64, 0);
    int32_t s_cap = 0, rows = 0;
    CHECK(ksa_cache_geometry(&p, &s_cap, &rows) == KSA_OK);
    std::vector<int> seen(rows);
    for (int64_t pos = 0; pos < n_cap; pos += (n_cap > 200 ? 7 : 1)) {
        int32_t rg[6];
        CHECK(ksa_decode_ranges(&p, pos, rg) == KSA_OK);
        std::fill(seen.begin(), seen.end(), 0);
        for (int x = 0; x < 3; ++x) {
            CHECK(rg[2 * x] >= 0 && rg[2 * x] + rg[2 * x + 1] <= rows);
            for (int r = rg[2 * x]; r < rg[2 * x] + rg[2 * x + 1]; ++r) seen[r] += 1;
        }
        // the rows read are exactly those of the visible tokens (Eq. 3), each once
        const int64_t j = pos / c, first = j - C > 0 ? j - C : 0;
        int want = 0;
        for (int64_t u = 0; u < first * m; ++u) {
            int32_t r;
            CHECK(ksa_cache_summary_row(&p, u, &r) == KSA_OK && seen[r] == 1);
            ++want;
        }
        for (int64_t i = first * c; i <= pos; ++i) {
            int32_t r;
            CHECK(ksa_cache_text_row(&p, i, &r) == KSA_OK && seen[r] == 1);
            ++want;
        }
        int got = 0;
        for (int r = 0; r < rows; ++r) got += seen[r];
        CHECK(got == want);
    }
    int32_t rg[6], r4[4];
    CHECK(ksa_decode_ranges(&p, n_cap, rg) == KSA_ERR_OUT_OF_RANGE);
    if (m > 0) CHECK(ksa_decode_summary_ranges(&p, s_cap - 1, r4) == KSA_OK);
    CHECK(ksa_decode_workspace_bytes(&p, 3) == (size_t)2 * 4 * 3 * 66 * 4);
    int dummy[64] = {0};
    CHECK(ksa_decode_fwd(&p, nullptr, dummy, dummy, dummy, dummy, nullptr, nullptr, dummy, 1 << 20, 0, nullptr) == KSA_ERR_INVALID_ARG);
    CHECK(ksa_decode_fwd(&p, dummy, dummy, dummy, dummy, dummy, nullptr, nullptr, dummy, 16, 3, nullptr) == KSA_ERR_WORKSPACE_TOO_SMALL);
    CHECK(ksa_decode_fwd_static(&p, dummy, dummy, dummy, dummy, dummy, nullptr, nullptr, 0, nullptr) == KSA_ERR_HIP);
    ksa_params big = make(4096, n_cap, c, m, C, 64, 8, 128, 0);
    CHECK(ksa_decode_fwd_static(&big, dummy, dummy, dummy, dummy, dummy, nullptr, nullptr, 16, nullptr) == KSA_ERR_SCRATCH_LIMIT);
    CHECK(ksa_cache_append(&p, 7, dummy, dummy, dummy, dummy, dummy, nullptr, nullptr) == KSA_ERR_INVALID_ARG);
    CHECK(ksa_cache_from_prefill(&p, n_cap + 1, dummy, dummy, nullptr, dummy, dummy, nullptr, nullptr) == KSA_ERR_OUT_OF_RANGE);
}

int main() {
    const int shapes[][5] = {{512, 64, 8, 1, 0}, {384, 64, 8, 0, 1}, {320, 64, 8, 9, 0}, {200, 8, 1, 3, 0}, {300, 20, 5, 1, 1},
                             {252, 12, 3, 2, 0}, {96, 96, 0, 0, 0}, {256, 16, 0, 2, 0}, {600, 64, 8, 1, 0}, {37, 64, 8, 1, 0},
                             {300, 1, 0, 40, 0}, {1003, 8, 1, 16, 0}};
    for (const auto &s : shapes) {
        layout_against_oracle(s[0], s[1], s[2], s[3], (unsigned)s[4], 4, 1);   // four heads stacked per workgroup
        layout_against_oracle(s[0], s[1], s[2], s[3], (unsigned)s[4], 2, 2);   // one head per workgroup
    }
    const int small[][5] = {{24, 4, 2, 1, 0}, {24, 4, 2, 1, 1}, {19, 4, 1, 2, 0}, {16, 16, 0, 0, 0}, {30, 1, 0, 6, 0}};
    for (const auto &s : small) oracle_numerics(s[0], s[1], s[2], s[3], (unsigned)s[4]);
    decode_checks(640, 64, 8, 1);
    decode_checks(96, 8, 1, 3);
    decode_checks(100, 1, 0, 15);
    ksa_params bad = make(1, 100, 64, 8, 1, 3, 2, 128, 0);
    ksa_layout *lay = nullptr;
    CHECK(ksa_build_layout(&bad, &lay) == KSA_ERR_INVALID_ARG && !lay);
    bad = make(1, 100, 64, 8, 1, 4, 2, 96, 0);
    CHECK(ksa_build_layout(&bad, &lay) == KSA_ERR_UNSUPPORTED && !lay);
    CHECK(ksa_build_layout(nullptr, &lay) == KSA_ERR_INVALID_ARG);
    std::printf("%s (%d failed checks)\n", failures ? "FAILED" : "host checks passed", failures);
    return failures ? 1 : 0;
}
