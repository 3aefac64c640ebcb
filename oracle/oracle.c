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
