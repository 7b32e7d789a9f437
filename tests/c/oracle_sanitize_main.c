/*
 * Driver for a sanitizer build of the CPU oracle (tests/test_oracle_sanitized.py compiles this file
 * together with oracle/mla_oracle.c under -fsanitize=address,undefined and runs it).  It calls every
 * entry point on small ragged inputs, including empty sequences, several query tokens and both
 * input types; any out-of-bounds access, leak or undefined operation makes the run fail.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int mla_oracle_decode(const uint16_t *, const uint16_t *, int64_t, const int32_t *, int, int, int, int, double,
                      double *, double *, int);
int mla_oracle_decode_general(const uint16_t *, const uint16_t *, int64_t, const int32_t *, int, int, int, int, int,
                              int, double, double *, double *, int);
int mla_oracle_decode_range(const uint16_t *, const uint16_t *, int64_t, const int32_t *, int, int, int, int, int,
                            int, double, double *, double *);
int mla_oracle_decode_transposed(const uint16_t *, const uint16_t *, int64_t, const int32_t *, int, int, int, int,
                                 double, double *, double *);
int mla_oracle_merge(const double *, const double *, int, int, double *, double *);
int mla_oracle_probs(const uint16_t *, const uint16_t *, int64_t, const int32_t *, int, int, int, int, double,
                     double *);

static uint32_t rng = 12345u;
static uint16_t small_bf16(void)
{   /* a bf16 in about [-2, 2]: sign, exponent 125..127, random fraction */
    rng = rng * 1664525u + 1013904223u;
    uint32_t r = rng >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((125u + (r >> 1) % 3u) << 7) | ((r >> 4) & 127u));
}
static uint16_t small_f16(void)
{
    rng = rng * 1664525u + 1013904223u;
    uint32_t r = rng >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((13u + (r >> 1) % 3u) << 10) | ((r >> 4) & 1023u));
}

int main(void)
{
    enum { B = 4, QL = 3, H = 5, D = 24, DV = 20, N = 37 };
    const int32_t lens[B] = {37, 0, 2, 1};
    uint16_t *q = malloc(sizeof(uint16_t) * B * QL * H * D);
    uint16_t *kv = malloc(sizeof(uint16_t) * B * N * D);
    double *out = malloc(sizeof(double) * B * QL * H * DV);
    double *lse = malloc(sizeof(double) * B * QL * H);
    double *p = malloc(sizeof(double) * N);
    if (!q || !kv || !out || !lse || !p) return 2;
    int bad = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        for (int i = 0; i < B * QL * H * D; ++i) q[i] = dtype ? small_f16() : small_bf16();
        for (int i = 0; i < B * N * D; ++i) kv[i] = dtype ? small_f16() : small_bf16();
        bad |= mla_oracle_decode_general(q, kv, (int64_t)N * D, lens, B, QL, H, D, DV, dtype, 0.3, out, lse, 3);
        for (int i = 0; i < B * QL * H * DV; ++i) bad |= isnan(out[i]);
    }
    /* bf16 entry points, one query token: q is read as [B][H][D] */
    bad |= mla_oracle_decode(q, kv, (int64_t)N * D, lens, B, H, D, DV, 0.3, out, lse, 2);
    bad |= mla_oracle_decode_transposed(q, kv, (int64_t)N * D, lens, B, H, D, DV, 0.3, out, lse);
    bad |= mla_oracle_decode_range(q, kv, (int64_t)N * D, lens, B, H, D, DV, 5, 19, 0.3, out, lse);
    bad |= mla_oracle_decode_range(q, kv, (int64_t)N * D, lens, B, H, D, DV, 30, 1000, 0.3, out, lse);
    bad |= mla_oracle_probs(q, kv, (int64_t)N * D, lens, H, D, 0, 2, 0.3, p);
    bad |= mla_oracle_probs(q, kv, (int64_t)N * D, lens, H, D, 1, 0, 0.3, p);      /* empty sequence */
    {
        double po[3 * DV], pl[3] = {0.5, -INFINITY, 2.0}, mo[DV], ml;
        for (int i = 0; i < 3 * DV; ++i) po[i] = 0.01 * i;
        bad |= mla_oracle_merge(po, pl, 3, DV, mo, &ml);
        pl[0] = pl[2] = -INFINITY;
        bad |= mla_oracle_merge(po, pl, 3, DV, mo, &ml);
        bad |= mla_oracle_merge(po, pl, 0, DV, mo, &ml);
    }
    /* argument errors return -1 and touch nothing */
    if (mla_oracle_decode(NULL, kv, 0, lens, B, H, D, DV, 0.3, out, lse, 1) != -1) bad = 1;
    if (mla_oracle_decode_general(q, kv, 0, lens, B, 0, H, D, DV, 0, 0.3, out, lse, 1) != -1) bad = 1;
    if (mla_oracle_decode_general(q, kv, 0, lens, B, 1, H, D, DV, 7, 0.3, out, lse, 1) != -1) bad = 1;
    free(q); free(kv); free(out); free(lse); free(p);
    printf(bad ? "FAILED\n" : "ok\n");
    return bad ? 1 : 0;
}
