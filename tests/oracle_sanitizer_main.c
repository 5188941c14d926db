/*
 * Driver for the address/undefined-behaviour sanitizer run of the C oracle (tests/test_oracle_sanitizer.py):
 * linked with oracle/kda_oracle.c under -fsanitize=address,undefined, it calls the forward and the backward
 * recurrence on exactly-sized heap buffers over the shapes that stress their indexing: ragged packed batches with
 * an empty sequence, tokens that belong to no sequence, a single token, no heads of work, NULL optional
 * arguments, and the malformed calls that must be refused before anything is touched.  Any access outside a
 * buffer aborts the run; the driver itself checks return codes and that the results are finite.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int kda_oracle_forward(int64_t B, int64_t T, int H, int dk, int dv, int64_t N, const float *q, const float *k,
                       const float *v, const float *log_alpha, const float *beta, const double *h0,
                       const int64_t *cu_seqlens, double scale, double *o, double *hT);
int kda_oracle_backward(int64_t B, int64_t T, int H, int dk, int dv, int64_t N, const float *q, const float *k,
                        const float *v, const float *log_alpha, const float *beta, const double *h0,
                        const int64_t *cu_seqlens, double scale, const double *d_o, const double *dhT, double *dq,
                        double *dk_out, double *dv_out, double *dla, double *dbeta, double *dh0);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static float *floats(size_t n, double lo, double hi)
{
    float *p = malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = (float)(lo + (hi - lo) * uniform());
    return p;
}
static double *doubles(size_t n, double lo, double hi)
{
    double *p = malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = lo + (hi - lo) * uniform();
    return p;
}
static int finite_all(const double *p, size_t n)
{
    for (size_t i = 0; i < n; ++i) if (!isfinite(p[i])) return 0;
    return 1;
}

/* one forward and one backward call; cu == NULL: B rows of T tokens */
static int run_case(const char *name, int64_t B, int64_t T, int H, int dk, int dv, int64_t N, const int64_t *cu,
                    int with_h0, int with_optional)
{
    const size_t tok = (size_t)B * T * H, st = (size_t)N * H * dk * dv;
    float *q = floats(tok * dk, -1, 1), *k = floats(tok * dk, -0.3, 0.3), *v = floats(tok * dv, -1, 1);
    float *la = floats(tok * dk, -0.5, 0.0), *beta = floats(tok, 0, 1);
    double *h0 = with_h0 ? doubles(st, -0.1, 0.1) : NULL;
    double *o = doubles(tok * dv, 0, 0), *hT = doubles(st, 0, 0);
    int rc = kda_oracle_forward(B, T, H, dk, dv, N, q, k, v, la, beta, h0, cu, 0.5, with_optional ? o : NULL,
                                with_optional ? hT : NULL);
    int ok = rc == 0 && (!with_optional || (finite_all(o, tok * dv) && finite_all(hT, st)));
    double *d_o = doubles(tok * dv, -1, 1), *dhT = with_optional ? doubles(st, -1, 1) : NULL;
    double *dq = doubles(tok * dk, 0, 0), *dkk = doubles(tok * dk, 0, 0), *dvv = doubles(tok * dv, 0, 0);
    double *dla = doubles(tok * dk, 0, 0), *db = doubles(tok, 0, 0), *dh0 = with_optional ? doubles(st, 0, 0) : NULL;
    rc = kda_oracle_backward(B, T, H, dk, dv, N, q, k, v, la, beta, h0, cu, 0.5, d_o, dhT, dq, dkk, dvv, dla, db, dh0);
    ok = ok && rc == 0 && finite_all(dq, tok * dk) && finite_all(dkk, tok * dk) && finite_all(dvv, tok * dv) &&
         finite_all(dla, tok * dk) && finite_all(db, tok) && (!dh0 || finite_all(dh0, st));
    printf("%-44s %s\n", name, ok ? "ok" : "FAILED");
    free(q); free(k); free(v); free(la); free(beta); free(h0); free(o); free(hT); free(d_o); free(dhT);
    free(dq); free(dkk); free(dvv); free(dla); free(db); free(dh0);
    return ok ? 0 : 1;
}

int main(void)
{
    int bad = 0;
    bad += run_case("batch 2 x 37 tokens, 3 heads, 8 x 4", 2, 37, 3, 8, 4, 2, NULL, 1, 1);
    bad += run_case("single token", 1, 1, 1, 4, 4, 1, NULL, 0, 1);
    bad += run_case("no tokens", 3, 0, 2, 4, 4, 3, NULL, 1, 1);
    bad += run_case("optional outputs left out", 1, 9, 2, 4, 8, 1, NULL, 0, 0);
    {   /* packed: lengths 5, 0, 11, 1 and three tokens after the last sequence */
        const int64_t cu[5] = {0, 5, 5, 16, 17};
        bad += run_case("packed, empty sequence, unowned tail tokens", 1, 20, 2, 8, 8, 4, cu, 1, 1);
    }
    {   const int64_t cu[1] = {0};
        bad += run_case("packed, no sequences", 1, 6, 2, 4, 4, 0, cu, 0, 1);
    }
    {   /* malformed calls: refused with a positive code, nothing written */
        float x[8] = {0}; double y[64] = {0};
        const int64_t down[3] = {0, 4, 2}, late[2] = {1, 2}, longer[2] = {0, 9};
        int ok = kda_oracle_forward(2, 2, 1, 2, 2, 1, x, x, x, x, x, NULL, NULL, 1.0, y, y) > 0;        /* N != B */
        ok = ok && kda_oracle_forward(2, 2, 1, 2, 2, 1, x, x, x, x, x, NULL, late, 1.0, y, y) > 0;      /* packed needs B == 1 */
        ok = ok && kda_oracle_forward(1, 4, 1, 2, 2, 2, x, x, x, x, x, NULL, down, 1.0, y, y) > 0;      /* decreasing offsets */
        ok = ok && kda_oracle_forward(1, 4, 1, 2, 2, 1, x, x, x, x, x, NULL, late, 1.0, y, y) > 0;      /* first offset not 0 */
        ok = ok && kda_oracle_forward(1, 4, 1, 2, 2, 1, x, x, x, x, x, NULL, longer, 1.0, y, y) > 0;    /* beyond T */
        ok = ok && kda_oracle_forward(1, 4, 0, 2, 2, 1, x, x, x, x, x, NULL, NULL, 1.0, y, y) > 0;      /* no heads */
        ok = ok && kda_oracle_backward(1, 4, 1, 2, 2, 2, x, x, x, x, x, NULL, down, 1.0, y, NULL, y, y, y, y, y, NULL) > 0;
        printf("%-44s %s\n", "malformed calls are refused", ok ? "ok" : "FAILED");
        bad += !ok;
    }
    return bad ? 1 : 0;
}
