// Host-only driver for the sanitizer test: exercises the CPU oracle (oracle/oracle.c) and the
// session prefix tree (csrc/prefix_tree.cpp) under AddressSanitizer and UBSan.  Test infrastructure:
// built and run by tests/test_host_sanitizers.py, never linked into the library.  Inputs come from a
// small linear congruential generator; checks are invariants that need no second implementation.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/seamdecode.h"

extern "C" {
float oracle_bf16_to_float(uint16_t bits);
float oracle_e4m3fn_to_float(uint8_t code);
uint8_t oracle_float_to_e4m3fn(float y);
void oracle_kv_append(int Hkv, int d, int max_blocks, int elem_bytes, const void *k_new, const void *v_new,
                      const int32_t *seq_ids, const int32_t *positions, int T, void *k_pages, void *v_pages,
                      const int32_t *block_table);
void oracle_kv_copy_pages(int num_pages, int Hkv, int d, int elem_bytes, const int32_t *src, const int32_t *dst, int n,
                          void *k_pages, void *v_pages, float *k_scales, float *v_scales);
void oracle_kv_append_fp8(int Hkv, int d, int max_blocks, const uint16_t *k_new, const uint16_t *v_new,
                          const int32_t *range_seq, const int32_t *range_start, const int32_t *range_row0, int R,
                          uint8_t *k_pages, uint8_t *v_pages, float *k_scales, float *v_scales, const int32_t *block_table);
int oracle_paged_decode_attention_f64(int B, int Hq, int Hkv, int d, int max_blocks, int kv_dtype, const uint16_t *q,
                                      const void *k_pages, const void *v_pages, const float *k_scales, const float *v_scales,
                                      const int32_t *block_table, const int32_t *context_lens, float scale, double *out);
int oracle_paged_decode_attention_f32(int B, int Hq, int Hkv, int d, int max_blocks, int kv_dtype, const uint16_t *q,
                                      const void *k_pages, const void *v_pages, const float *k_scales, const float *v_scales,
                                      const int32_t *block_table, const int32_t *context_lens, float scale, float *out);
int oracle_partial_f64(int Hq, int Hkv, int d, int max_blocks, int kv_dtype, const uint16_t *q, const void *k_pages,
                       const void *v_pages, const float *k_scales, const float *v_scales, const int32_t *block_table,
                       float scale, int b, int h, int t0, int t1, double *m, double *l, double *acc);
void oracle_combine_f64(int n, int d, const double *m, const double *l, const double *acc, double *out);
int oracle_paged_prefill_attention_f64(int B, int Hq, int Hkv, int d, int max_blocks, int kv_dtype, const uint16_t *q,
                                       const int32_t *q_start, const void *k_pages, const void *v_pages,
                                       const float *k_scales, const float *v_scales, const int32_t *block_table,
                                       const int32_t *context_lens, float scale, double *out);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd()
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33);
}
static int rnd_int(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
// a bf16 bit pattern of a value in about [-4, 4]
static uint16_t rnd_bf16()
{
    const float v = ((int)(rnd() % 2001) - 1000) / 250.0f;
    uint32_t w;
    memcpy(&w, &v, 4);
    return (uint16_t)(w >> 16);
}
#define CHECK(c)                                                                  \
    do {                                                                          \
        if (!(c)) {                                                               \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c);       \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

static void oracle_cases(int kv_fp8)
{
    const int B = 5, Hq = 8, Hkv = 2, d = 64, P = 16;
    const int lens[B] = {1, 40, 0, 129, 16};
    int maxnb = 0, total = 0;
    for (int b = 0; b < B; ++b) {
        const int nb = (lens[b] + P - 1) / P;
        maxnb = nb > maxnb ? nb : maxnb;
        total += nb;
    }
    const int num_pages = total + 3;
    // a fixed permutation of the pages: logical page j of the whole batch -> (7 * j + 3) mod num_pages
    std::vector<int32_t> table((size_t)B * maxnb, -1), clen(lens, lens + B);
    int next = 0;
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < (lens[b] + P - 1) / P; ++j) table[(size_t)b * maxnb + j] = (7 * next++ + 3) % num_pages;
    const size_t tile = (size_t)P * d, pool = (size_t)num_pages * Hkv * tile;
    std::vector<uint16_t> q((size_t)B * Hq * d);
    for (auto &x : q) x = rnd_bf16();
    const float scale = 0.125f;
    std::vector<double> out((size_t)B * Hq * d), out2(out.size());
    std::vector<float> out32(out.size());
    if (!kv_fp8) {
        std::vector<uint16_t> k(pool, 0x7FC0), v(pool, 0x7FC0);  // NaN everywhere; valid slots are appended below
        int T = 0;
        for (int b = 0; b < B; ++b) T += lens[b];
        std::vector<uint16_t> kn((size_t)T * Hkv * d), vn(kn.size());
        std::vector<int32_t> seq(T), pos(T);
        for (auto &x : kn) x = rnd_bf16();
        for (auto &x : vn) x = rnd_bf16();
        for (int b = 0, t = 0; b < B; ++b)
            for (int p = 0; p < lens[b]; ++p, ++t) seq[t] = b, pos[t] = p;
        oracle_kv_append(Hkv, d, maxnb, 2, kn.data(), vn.data(), seq.data(), pos.data(), T, k.data(), v.data(), table.data());
        CHECK(oracle_paged_decode_attention_f64(B, Hq, Hkv, d, maxnb, 0, q.data(), k.data(), v.data(), nullptr, nullptr,
                                                table.data(), clen.data(), scale, out.data()) == 0);
        CHECK(oracle_paged_decode_attention_f32(B, Hq, Hkv, d, maxnb, 0, q.data(), k.data(), v.data(), nullptr, nullptr,
                                                table.data(), clen.data(), scale, out32.data()) == 0);
        for (size_t i = 0; i < out.size(); ++i) CHECK(std::isfinite(out[i]) && std::fabs(out[i] - out32[i]) < 1e-4);
        // a context of one token returns its V row; an empty one zeros
        for (int h = 0; h < Hq; ++h)
            for (int i = 0; i < d; ++i) {
                CHECK(out[(0 * Hq + h) * d + i] == oracle_bf16_to_float(vn[(size_t)(h / (Hq / Hkv)) * d + i]));
                CHECK(out[(2 * Hq + h) * d + i] == 0.0);
            }
        // split at an arbitrary token and merge: the identity the GPU method relies on
        std::vector<double> m(2), l(2), acc(2 * d), merged(d);
        CHECK(oracle_partial_f64(Hq, Hkv, d, maxnb, 0, q.data(), k.data(), v.data(), nullptr, nullptr, table.data(), scale, 3, 5, 0, 50,
                                 &m[0], &l[0], &acc[0]) == 0);
        CHECK(oracle_partial_f64(Hq, Hkv, d, maxnb, 0, q.data(), k.data(), v.data(), nullptr, nullptr, table.data(), scale, 3, 5, 50, 129,
                                 &m[1], &l[1], &acc[d]) == 0);
        oracle_combine_f64(2, d, m.data(), l.data(), acc.data(), merged.data());
        for (int i = 0; i < d; ++i) CHECK(std::fabs(merged[i] - out[(3 * Hq + 5) * d + i]) < 1e-9);
        // causal pass: one query per sequence is the decode step
        std::vector<int32_t> qs(B + 1);
        for (int b = 0; b <= B; ++b) qs[b] = b;
        CHECK(oracle_paged_prefill_attention_f64(B, Hq, Hkv, d, maxnb, 0, q.data(), qs.data(), k.data(), v.data(), nullptr, nullptr,
                                                 table.data(), clen.data(), scale, out2.data()) == 0);
        for (size_t i = 0; i < out.size(); ++i) CHECK(out[i] == out2[i]);
        // copy a page onto a spare one and read through the copy
        const int32_t src = table[(size_t)1 * maxnb + 1], dst = (7 * next + 3) % num_pages;
        oracle_kv_copy_pages(num_pages, Hkv, d, 2, &src, &dst, 1, k.data(), v.data(), nullptr, nullptr);
        table[(size_t)1 * maxnb + 1] = dst;
        CHECK(oracle_paged_decode_attention_f64(B, Hq, Hkv, d, maxnb, 0, q.data(), k.data(), v.data(), nullptr, nullptr,
                                                table.data(), clen.data(), scale, out2.data()) == 0);
        for (size_t i = 0; i < out.size(); ++i) CHECK(out[i] == out2[i]);
    } else {
        std::vector<uint8_t> k(pool, 0x7F), v(pool, 0x7F);
        std::vector<float> ks((size_t)num_pages * Hkv, NAN), vs(ks.size(), NAN);
        // every sequence in three ranges: a fresh one, one that continues inside a page with small values (scale
        // stays), one with large values (scale grows and old codes are re-encoded)
        for (int b = 0; b < B; ++b) {
            const int cuts[4] = {0, lens[b] / 3, 2 * lens[b] / 3, lens[b]};
            for (int part = 0; part < 3; ++part) {
                const int n = cuts[part + 1] - cuts[part];
                if (n <= 0) continue;
                std::vector<uint16_t> kn((size_t)n * Hkv * d), vn(kn.size());
                for (auto &x : kn) x = rnd_bf16();
                for (auto &x : vn) x = rnd_bf16();
                if (part == 1)
                    for (auto &x : kn) x = (uint16_t)(x & 0x8000) | 0x3C00;  // +-2^-7: never raises a scale
                if (part == 2) kn[0] = 0x4300, vn[0] = 0xC300;                // +-128: raises it
                const int32_t rs = b, st = cuts[part], r0[2] = {0, n};
                oracle_kv_append_fp8(Hkv, d, maxnb, kn.data(), vn.data(), &rs, &st, r0, 1, k.data(), v.data(), ks.data(), vs.data(),
                                     table.data());
            }
        }
        CHECK(oracle_paged_decode_attention_f64(B, Hq, Hkv, d, maxnb, 1, q.data(), k.data(), v.data(), ks.data(), vs.data(),
                                                table.data(), clen.data(), scale, out.data()) == 0);
        for (size_t i = 0; i < out.size(); ++i) CHECK(std::isfinite(out[i]));
        for (int c = 0; c < 256; ++c) {   // the encoder inverts the decoder on every finite code
            const float f = oracle_e4m3fn_to_float((uint8_t)c);
            if (std::isnan(f)) continue;
            CHECK(oracle_float_to_e4m3fn(f) == (uint8_t)c);
        }
    }
}

// a random session on the prefix tree; every answer is checked against the token lists kept here
static void tree_session()
{
    sd_tree *t = sd_tree_create(512);
    CHECK(t != nullptr);
    std::vector<std::vector<int32_t>> toks;
    std::vector<int32_t> ids;
    for (int step = 0; step < 300; ++step) {
        const int op = ids.empty() ? 0 : rnd_int(0, 9);
        if (op <= 2) {   // insert: a fresh trajectory or a continuation of a stored prefix
            std::vector<int32_t> tr;
            if (!toks.empty() && rnd_int(0, 1)) {
                const auto &src = toks[rnd_int(0, (int)toks.size() - 1)];
                tr.assign(src.begin(), src.begin() + rnd_int(1, (int)src.size()));
            }
            for (int n = rnd_int(1, 60); n > 0; --n) tr.push_back(rnd_int(0, 3));
            const int32_t want = sd_tree_match(t, tr.data(), nullptr, (int32_t)tr.size());
            int32_t matched = -1;
            const int32_t id = sd_tree_insert(t, tr.data(), nullptr, (int32_t)tr.size(), &matched);
            if (id == SD_EWORKSPACE) continue;   // pool exhausted: nothing stored
            CHECK(id >= 0 && matched == want && matched % 16 == 0 && (size_t)matched <= tr.size());
            CHECK(sd_tree_length(t, id) == (int32_t)tr.size());
            toks.push_back(tr);
            ids.push_back(id);
        } else if (op <= 4) {   // fork
            const int s = rnd_int(0, (int)ids.size() - 1);
            if (ids[s] < 0) continue;
            int32_t cs = -2, cd = -2;
            const int32_t id = sd_tree_fork(t, ids[s], &cs, &cd);
            if (id == SD_EWORKSPACE) continue;
            CHECK(id >= 0 && ((cs == -1 && cd == -1) || (cs >= 0 && cd >= 0 && cs != cd)));
            CHECK((toks[s].size() % 16 == 0) == (cs == -1));
            toks.push_back(toks[s]);
            ids.push_back(id);
        } else if (op <= 7) {   // append
            const int s = rnd_int(0, (int)ids.size() - 1);
            if (ids[s] < 0) continue;
            int32_t page = -1, slot = -1;
            const int32_t tok = rnd_int(0, 3);
            const int rc = sd_tree_append(t, ids[s], tok, 0, &page, &slot);
            if (rc == SD_EWORKSPACE) continue;
            CHECK(rc == SD_OK && page >= 0 && page < 512 && slot == (int32_t)(toks[s].size() % 16));
            toks[s].push_back(tok);
        } else if (op == 8) {   // release
            const int s = rnd_int(0, (int)ids.size() - 1);
            if (ids[s] < 0) continue;
            CHECK(sd_tree_release(t, ids[s]) == SD_OK);
            ids[s] = -1;
        } else {   // read back: tokens, tables, groups
            std::vector<int32_t> live;
            for (size_t s = 0; s < ids.size(); ++s) {
                if (ids[s] < 0) continue;
                live.push_back(ids[s]);
                int32_t tok = -1;
                uint32_t ver = 9;
                const int32_t pos = rnd_int(0, (int)toks[s].size() - 1);
                CHECK(sd_tree_token_at(t, ids[s], pos, &tok, &ver) == SD_OK && tok == toks[s][pos] && ver == 0);
                std::vector<int32_t> pages(toks[s].size() / 16 + 2, -7);
                const int32_t np = sd_tree_block_table(t, ids[s], pages.data(), (int32_t)pages.size());
                CHECK(np == (int32_t)((toks[s].size() + 15) / 16));
                for (int j = 0; j < np; ++j) CHECK(pages[j] >= 0 && pages[j] < 512);
            }
            if (!live.empty()) {
                std::vector<int32_t> gs(live.size() + 1), sh(live.size());
                const int32_t ng = sd_tree_batch_groups(t, live.data(), (int32_t)live.size(), gs.data(), sh.data());
                CHECK(ng >= 1 && ng <= (int32_t)live.size() && gs[0] == 0 && gs[ng] == (int32_t)live.size());
                for (size_t i = 0; i < live.size(); ++i) CHECK(sh[i] >= 0 && sh[i] % 16 == 0);
            }
        }
    }
    CHECK(sd_tree_pages_in_use(t) >= 0 && sd_tree_pages_in_use(t) <= 512);
    sd_tree_destroy(t);
}

int main()
{
    oracle_cases(0);
    oracle_cases(1);
    tree_session();
    printf("host sanitizer driver: OK\n");
    return 0;
}
