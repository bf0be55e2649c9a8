/*
 * sanitize_main.c -- drives the CPU oracle (slicer_ref.c) under AddressSanitizer and
 * UndefinedBehaviorSanitizer.  TEST INFRASTRUCTURE ONLY: built and run by
 * tests/test_oracle_sanitizers.py as
 *   gcc -O1 -g -std=c11 -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan
 *       -ffp-contract=off -fopenmp oracle/sanitize_main.c oracle/slicer_ref.c -lm
 * It encodes and decodes small tensors of both dtypes in every mode (budget search, DS guard,
 * fixed ladder, asymmetric thresholds, separate block counts), including the degenerate shapes
 * (one element, k = 0, k = N, all zero, all equal, more blocks than entries), with one and
 * with several threads, and checks only that the calls succeed and agree between thread
 * counts: the sanitizers do the rest.  Inputs come from a small linear congruential generator.
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "slicer_ref.h"

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state >> 8; }

static float sample(int kind)
{
    float u = (float)(lcg() % 20001) / 10000.0f - 1.0f;          /* [-1, 1] */
    if (kind == 1) return 0.0f;                                    /* all zero */
    if (kind == 2) return 1.5f;                                    /* all equal */
    if (kind == 3) return (lcg() % 3) ? 0.0f : u;                  /* many zeros */
    if (kind == 4) return (float)((int)(lcg() % 7) - 3) * 0.25f;   /* heavy ties */
    if (kind == 5) return u * 1e-39f;                              /* denormals */
    return u * (lcg() % 50 == 0 ? 30.0f : 1.0f);                   /* outliers */
}

static uint16_t to_bf16_trunc(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16); }

static int run_case(int dt, int64_t R, int64_t N, double keep, int M, int Mn, int kind)
{
    const size_t esz = dt == SLICER_REF_F32 ? 4 : 2;
    void* x = malloc((size_t)(R * N) * esz);
    for (int64_t i = 0; i < R * N; ++i) {
        float v = sample(kind);
        if (dt == SLICER_REF_F32) ((float*)x)[i] = v; else ((uint16_t*)x)[i] = to_bf16_trunc(v);
    }
    const uint32_t bits = 0x1FCu;                                   /* {2..8} */
    size_t cap = 0, mb = 0, cap2 = 0, mb2 = 0;
    if (slicer_ref_sizes_pn(dt, R, N, keep, M, Mn, bits, &cap, &mb)) return 1;
    if (slicer_ref_sizes(dt, R, N, keep, M, bits | (1u << 16), &cap2, &mb2)) return 1;   /* the modes with one block count */
    if (cap2 > cap) cap = cap2;
    if (mb2 > mb) mb = mb2;
    int bad = 0;
    for (int mode = 0; mode < 5 && !bad; ++mode) {
        void* s[2]; void* m[2]; void* y[2];
        for (int t = 0; t < 2 && !bad; ++t) {
            s[t] = calloc(cap / 4 + 1, 4); m[t] = calloc(mb, 1); y[t] = malloc((size_t)(R * N) * esz);
            const int nt = t ? 3 : 1;
            int rc;
            uint8_t ladder[64];
            for (int j = 0; j < 64; ++j) ladder[j] = (uint8_t)(8 - (j % 7));
            if (mode == 0) rc = slicer_ref_encode_pn(x, dt, R, N, keep, M, Mn, bits, 1e-3, s[t], m[t], nt);
            else if (mode == 1) rc = slicer_ref_encode_ds(x, dt, R, N, keep, M, bits, 0.3, s[t], m[t], nt);
            else if (mode == 2) rc = slicer_ref_encode_ladder(x, dt, R, N, keep, M, ladder, s[t], m[t], nt);
            else if (mode == 3) rc = slicer_ref_encode_atkf(x, dt, R, N, keep, 0.25, M, Mn, bits, 1e-3, s[t], m[t], nt);
            else rc = slicer_ref_encode(x, dt, R, N, keep, M, 1u << 16, 0.0, s[t], m[t], nt);
            if (rc) { bad = 1; break; }
            if (slicer_ref_decode(s[t], m[t], y[t], nt)) { bad = 1; break; }
        }
        if (!bad && (memcmp(m[0], m[1], mb) || memcmp(s[0], s[1], cap) || memcmp(y[0], y[1], (size_t)(R * N) * esz))) bad = 2;
        for (int t = 0; t < 2; ++t) { free(s[t]); free(m[t]); free(y[t]); }
    }
    free(x);
    if (bad) fprintf(stderr, "case dt=%d R=%lld N=%lld keep=%g M=%d Mn=%d kind=%d: %s\n", dt, (long long)R,
                     (long long)N, keep, M, Mn, kind, bad == 2 ? "thread counts disagree" : "call failed");
    return bad;
}

int main(void)
{
    static const int64_t Ns[] = { 1, 2, 7, 64, 333, 1024 };
    static const double keeps[] = { 0.0, 0.1, 0.5, 1.0 };
    int bad = 0, n = 0;
    for (int dt = 0; dt < 2; ++dt)
        for (size_t a = 0; a < sizeof Ns / sizeof *Ns; ++a)
            for (size_t b = 0; b < sizeof keeps / sizeof *keeps; ++b)
                for (int kind = 0; kind < 6; ++kind) {
                    const int M = 1 + (int)((a + b + (size_t)kind) % 8), Mn = 1 + (int)((a * 3 + b) % 5);
                    bad |= run_case(dt, 1 + (int64_t)(kind % 3) * 2, Ns[a], keeps[b], M, Mn, kind);
                    ++n;
                }
    /* analysis view of one row, with and without the inspection arrays */
    {
        float row[100]; int32_t blk[100]; uint32_t code[100]; float vmin[8], vmax[8]; uint8_t qb[8];
        uint64_t s_int[8 * 17], e_int[8]; int32_t e_exp[8];
        for (int i = 0; i < 100; ++i) row[i] = sample(0);
        bad |= slicer_ref_analyze_row(row, SLICER_REF_F32, 100, 0.4, 4, 0x1FCu, 1e-3, blk, code, vmin, vmax, qb, s_int, e_int, e_exp);
        bad |= slicer_ref_analyze_row_atkf(row, SLICER_REF_F32, 100, 0.4, 0.5, 4, 0x1FCu, 1e-3, blk, code, vmin, vmax, qb);
    }
    printf("%d cases, %s\n", n, bad ? "FAILED" : "clean");
    return bad ? 1 : 0;
}
