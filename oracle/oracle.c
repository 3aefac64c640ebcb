/*
 * CPU oracle for paged decode attention and KV append.
 *
 * TEST INFRASTRUCTURE ONLY: plain, slow, written from the definition.  It is
 * called by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, and by nothing else.  It shares no code, header, table or constant
 * with the GPU library.
 *
 * Context in the paper: rollout (System Overview, inference-engine layer) is
 * batched autoregressive decoding; partial rollout (Data Plane, Rollout
 * Manager / Trajectory Manager paragraphs) pauses and resumes sequences from
 * their stored tokens, and one session may branch into several trajectories
 * over a common prefix.  The paper gives no formula for the decode step; the
 * step is the textbook one written out in oracle_attention_impl.h.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC oracle.c -o liboracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_PAGE 16
#define ORACLE_KV_BF16 0
#define ORACLE_KV_FP8_E4M3FN 1

/* bf16 = the upper 16 bits of an IEEE binary32 word */
float oracle_bf16_to_float(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

/*
 * OCP 8-bit float, E4M3 "fn" flavour: 1 sign, 4 exponent (bias 7), 3 mantissa
 * bits; no infinities; S.1111.111 is NaN; exponent field 0 is subnormal.
 * Largest finite value: 1.75 * 2^8 = 448.
 */
float oracle_e4m3fn_to_float(uint8_t code)
{
    int sign = code >> 7, e = (code >> 3) & 0xF, m = code & 0x7;
    float v;
    if (e == 0xF && m == 0x7)
        v = NAN;
    else if (e == 0)
        v = ldexpf((float)m / 8.0f, -6);
    else
        v = ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return sign ? -v : v;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * KV append (resuming or advancing a rollout writes the new tokens' K/V rows
 * into their page slots): row j of k_new/v_new [T][Hkv][d] belongs to
 * sequence seq_ids[j] at position positions[j] and goes to page
 * block_table[seq][pos/16], slot pos%16, for every KV head.  elem_bytes is
 * the size of one stored element (2 for bf16).  Plain copy, no conversion.
 */
void oracle_kv_append(int Hkv, int d, int max_blocks, int elem_bytes,
                      const void *k_new, const void *v_new,
                      const int32_t *seq_ids, const int32_t *positions, int T,
                      void *k_pages, void *v_pages, const int32_t *block_table)
{
    size_t row = (size_t)d * (size_t)elem_bytes;
    for (int j = 0; j < T; ++j) {
        int64_t page = block_table[(int64_t)seq_ids[j] * max_blocks + positions[j] / ORACLE_PAGE];
        int slot = positions[j] % ORACLE_PAGE;
        for (int g = 0; g < Hkv; ++g) {
            size_t dst = ((((size_t)page * Hkv + g) * ORACLE_PAGE) + slot) * row;
            size_t src = ((size_t)j * Hkv + g) * row;
            memcpy((char *)k_pages + dst, (const char *)k_new + src, row);
            memcpy((char *)v_pages + dst, (const char *)v_new + src, row);
        }
    }
}

/*
 * Whole-page copy inside the pool (a branch of a session whose last page is
 * partly filled gets a private copy of that page): for each pair, every byte
 * of page src -- all KV heads, K and V -- and, when the pool has scales, its
 * Hkv scales go to page dst.  Pairs are taken in order; a pair with an id
 * outside [0, num_pages) or with src == dst does nothing.
 */
void oracle_kv_copy_pages(int num_pages, int Hkv, int d, int elem_bytes,
                          const int32_t *src_pages, const int32_t *dst_pages, int n,
                          void *k_pages, void *v_pages, float *k_scales, float *v_scales)
{
    size_t page = (size_t)Hkv * ORACLE_PAGE * (size_t)d * (size_t)elem_bytes;
    for (int i = 0; i < n; ++i) {
        int s = src_pages[i], t = dst_pages[i];
        if (s < 0 || t < 0 || s >= num_pages || t >= num_pages || s == t) continue;
        memcpy((char *)k_pages + (size_t)t * page, (const char *)k_pages + (size_t)s * page, page);
        memcpy((char *)v_pages + (size_t)t * page, (const char *)v_pages + (size_t)s * page, page);
        if (k_scales && v_scales)
            for (int g = 0; g < Hkv; ++g) {
                k_scales[(size_t)t * Hkv + g] = k_scales[(size_t)s * Hkv + g];
                v_scales[(size_t)t * Hkv + g] = v_scales[(size_t)s * Hkv + g];
            }
    }
}

#define REAL double
#define REAL_EXP exp
#define NAME(x) x##_f64
#include "oracle_attention_impl.h"
#undef REAL
#undef REAL_EXP
#undef NAME

#define REAL float
#define REAL_EXP expf
#define NAME(x) x##_f32
#include "oracle_attention_impl.h"
#undef REAL
#undef REAL_EXP
#undef NAME

/*
 * Quantising append into fp8 pools (resuming a paused trajectory rewrites the
 * KV of its stored tokens; with an fp8 cache the rows must be quantised as
 * they are written).
 *
 * Encoding: nearest OCP e4m3fn value, ties to the even code, magnitudes above
 * 448 saturate to 448; the sign is kept (also for zero).
 */
uint8_t oracle_float_to_e4m3fn(float y)
{
    uint8_t sign = signbit(y) ? 0x80 : 0;
    float a = fabsf(y);
    if (isnan(a)) return sign | 0x7F;
    if (a >= 448.0f) return sign | 0x7E;
    /* candidates are the 127 finite magnitudes, ascending with the code */
    int best = 0;
    float best_err = a; /* distance to code 0 */
    for (int c = 1; c <= 0x7E; ++c) {
        float v = oracle_e4m3fn_to_float((uint8_t)c);
        float err = fabsf(v - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best = c;
            best_err = err;
        }
    }
    return sign | (uint8_t)best;
}

/*
 * One range of consecutive positions of one sequence: rows row0 .. row0+n-1 of
 * k_new/v_new ([T][Hkv][d] bf16) go to positions start .. start+n-1.  Per
 * (page, kv head) tile touched, for K and for V alike:
 *   s0 = first slot written (slots below it hold earlier tokens of the sequence
 *        when the range starts inside the page; a range that starts a page
 *        treats the page as fresh and ignores its old scale)
 *   amax_new = max |x| over the rows written into the tile
 *   old_amax = old_scale * 448 if s0 > 0 else 0
 *   if amax_new <= old_amax: scale stays, old codes stay
 *   else: scale = amax_new / 448 (fp32); each old code c in slots < s0 becomes
 *         enc(dec(c) * (old_scale / scale)), all in fp32: one ratio per tile
 *   fresh tile with amax_new == 0: scale = 1
 *   new codes: enc(x / scale) in fp32.
 */
void oracle_kv_append_fp8(int Hkv, int d, int max_blocks,
                          const uint16_t *k_new, const uint16_t *v_new,
                          const int32_t *range_seq, const int32_t *range_start,
                          const int32_t *range_row0, int R,
                          uint8_t *k_pages, uint8_t *v_pages, float *k_scales, float *v_scales,
                          const int32_t *block_table)
{
    for (int r = 0; r < R; ++r) {
        int seq = range_seq[r], start = range_start[r];
        int n = range_row0[r + 1] - range_row0[r];
        int end = start + n;
        for (int pg = start / ORACLE_PAGE; pg * ORACLE_PAGE < end; ++pg) {
            int64_t page = block_table[(int64_t)seq * max_blocks + pg];
            int p0 = pg * ORACLE_PAGE;
            int s0 = start > p0 ? start - p0 : 0;
            int s1 = end < p0 + ORACLE_PAGE ? end - p0 : ORACLE_PAGE;
            for (int g = 0; g < Hkv; ++g) {
                for (int which = 0; which < 2; ++which) {
                    const uint16_t *src = which ? v_new : k_new;
                    uint8_t *tile = (which ? v_pages : k_pages) + ((int64_t)page * Hkv + g) * ORACLE_PAGE * d;
                    float *scale_p = (which ? v_scales : k_scales) + (int64_t)page * Hkv + g;
                    float amax_new = 0.0f;
                    for (int s = s0; s < s1; ++s) {
                        const uint16_t *row = src + ((int64_t)(range_row0[r] + p0 + s - start) * Hkv + g) * d;
                        for (int i = 0; i < d; ++i) {
                            float a = fabsf(oracle_bf16_to_float(row[i]));
                            if (a > amax_new) amax_new = a;
                        }
                    }
                    float old_scale = s0 > 0 ? *scale_p : 0.0f;
                    float old_amax = old_scale * 448.0f;
                    float scale;
                    if (s0 > 0 && amax_new <= old_amax) {
                        scale = old_scale;
                    } else {
                        scale = amax_new > 0.0f ? amax_new / 448.0f : 1.0f;
                        float ratio = old_scale / scale;
                        for (int s = 0; s < s0; ++s)
                            for (int i = 0; i < d; ++i)
                                tile[s * d + i] = oracle_float_to_e4m3fn(oracle_e4m3fn_to_float(tile[s * d + i]) * ratio);
                        *scale_p = scale;
                    }
                    for (int s = s0; s < s1; ++s) {
                        const uint16_t *row = src + ((int64_t)(range_row0[r] + p0 + s - start) * Hkv + g) * d;
                        for (int i = 0; i < d; ++i)
                            tile[s * d + i] = oracle_float_to_e4m3fn(oracle_bf16_to_float(row[i]) / scale);
                    }
                }
            }
        }
    }
}
