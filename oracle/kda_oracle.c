/*
 * kda_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain fp64 CPU oracle for Kimi Delta Attention (KDA).  It evaluates the
 * defining per-token recurrence of the paper's Section 3, Eq. (1)
 *
 *     S_t = (I - beta_t k_t k_t^T) Diag(alpha_t) S_{t-1} + beta_t k_t v_t^T
 *     o_t = S_t^T q_t
 *
 * literally, one token at a time, with no chunking, no fusion and no
 * reordering beyond what the equation states.  The chunkwise algorithm of
 * Section 3.1 reaches this same result (up to rounding order), so this file is
 * the definition written out.  It shares no code with the HIP path and may be
 * used only by tests, the smoke check and the CPU-baseline leg of the bench.
 *
 * Readings of the paper taken here (all documented with the design notes):
 *   - alpha_t = exp(log_alpha_t), natural logarithm, per key channel.
 *   - Order inside a step: decay first, then the Householder-style
 *     correction, then the un-decayed write beta k v^T (Section 6.1 "Relation
 *     to DPLR": decay "followed by" the Householder transform).
 *   - o_t reads the UPDATED state S_t.
 *   - `scale` multiplies o (1.0 reproduces Eq. (1); the App. C listing folds
 *     d_k^-1/2 into q, which is the same thing by linearity).
 *   - Packed batches: sequence n owns tokens [cu[n], cu[n+1]) of the single
 *     token stream; every sequence starts from its own h0 (zeros if absent).
 *
 * Inputs are float32 arrays because every bf16 and fp32 value the GPU path
 * receives is exactly representable in float32; they are widened to double
 * before any arithmetic.  State, accumulation and outputs are double.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC -o libkda_oracle.so kda_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the parallel region will use (reported by the bench). */
int kda_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One (sequence, head) pair: run tokens [t0, t1) of batch row `row`.
 * Token (row, t), head h lives at ((row*T + t)*H + h) in the [B,T,H,*] arrays.
 */
static void run_sequence(int64_t row, int64_t t0, int64_t t1, int64_t T, int H, int h,
                         int dk, int dv,
                         const float *q, const float *k, const float *v,
                         const float *log_alpha, const float *beta,
                         double scale, double *S /* [dk,dv], in/out */,
                         double *o /* [B,T,H,dv] or NULL */)
{
    double *kd = (double *)malloc(sizeof(double) * (size_t)(3 * dk + 2 * dv));
    double *qd = kd + dk, *ad = qd + dk, *vd = ad + dk, *r = vd + dv;

    for (int64_t t = t0; t < t1; ++t) {
        const int64_t tok = (row * T + t) * H + h;
        for (int i = 0; i < dk; ++i) {
            kd[i] = (double)k[tok * dk + i];
            qd[i] = (double)q[tok * dk + i];
            ad[i] = exp((double)log_alpha[tok * dk + i]);   /* alpha_t, per channel */
        }
        for (int j = 0; j < dv; ++j) vd[j] = (double)v[tok * dv + j];
        const double b = (double)beta[tok];

        /* S <- Diag(alpha_t) S_{t-1} */
        for (int i = 0; i < dk; ++i)
            for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] *= ad[i];

        /* r = v_t - S^T k_t   (prediction error of the decayed memory) */
        for (int j = 0; j < dv; ++j) r[j] = 0.0;
        for (int i = 0; i < dk; ++i)
            for (int j = 0; j < dv; ++j) r[j] += kd[i] * S[(size_t)i * dv + j];
        for (int j = 0; j < dv; ++j) r[j] = vd[j] - r[j];

        /* S <- S + beta_t k_t r^T  ==  (I - beta k k^T) S + beta k v^T */
        for (int i = 0; i < dk; ++i) {
            const double bk = b * kd[i];
            for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] += bk * r[j];
        }

        /* o_t = scale * S_t^T q_t */
        if (o) {
            double *ot = o + tok * dv;
            for (int j = 0; j < dv; ++j) ot[j] = 0.0;
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j) ot[j] += qd[i] * S[(size_t)i * dv + j];
            for (int j = 0; j < dv; ++j) ot[j] *= scale;
        }
    }
    free(kd);
}

/*
 * Whole forward pass.
 *   q,k,log_alpha : [B,T,H,dk]   v : [B,T,H,dv]   beta : [B,T,H]   (float32)
 *   h0            : [N,H,dk,dv] double, or NULL for zeros
 *   cu_seqlens    : [N+1] int64 token offsets into the T axis (requires B==1),
 *                   or NULL, in which case N must equal B and sequence n is
 *                   batch row n, tokens [0,T)
 *   o             : [B,T,H,dv] double (may be NULL)
 *   hT            : [N,H,dk,dv] double (may be NULL)
 * Returns 0 on success, a positive code on a malformed call.
 */
int kda_oracle_forward(int64_t B, int64_t T, int H, int dk, int dv, int64_t N,
                       const float *q, const float *k, const float *v,
                       const float *log_alpha, const float *beta,
                       const double *h0, const int64_t *cu_seqlens,
                       double scale, double *o, double *hT)
{
    if (B < 0 || T < 0 || H <= 0 || dk <= 0 || dv <= 0 || N < 0) return 1;
    if (cu_seqlens) {
        if (B != 1) return 2;
        if (cu_seqlens[0] != 0 || cu_seqlens[N] > T) return 3;
        for (int64_t n = 0; n < N; ++n)
            if (cu_seqlens[n + 1] < cu_seqlens[n]) return 3;
    } else if (N != B) {
        return 4;
    }

    const int64_t pairs = N * (int64_t)H;
    const size_t ssz = (size_t)dk * dv;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < pairs; ++p) {
        const int64_t n = p / H;
        const int h = (int)(p % H);
        double *S = (double *)malloc(sizeof(double) * ssz);
        if (h0) memcpy(S, h0 + (size_t)p * ssz, sizeof(double) * ssz);
        else    memset(S, 0, sizeof(double) * ssz);

        int64_t row, t0, t1;
        if (cu_seqlens) { row = 0; t0 = cu_seqlens[n]; t1 = cu_seqlens[n + 1]; }
        else            { row = n; t0 = 0;             t1 = T; }

        run_sequence(row, t0, t1, T, H, h, dk, dv, q, k, v, log_alpha, beta, scale, S, o);

        if (hT) memcpy(hT + (size_t)p * ssz, S, sizeof(double) * ssz);
        free(S);
    }
    return 0;
}
