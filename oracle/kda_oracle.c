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

/*
 * ---------------------------------------------------------------------------
 * Backward pass: reverse-mode differentiation of Eq. (1), token by token.
 *
 * The paper motivates a training kernel but derives no backward algorithm, so
 * the definition is the chain rule applied to the recurrence as written above.
 * With  S' = Diag(alpha_t) S_{t-1},  u = v_t - S'^T k_t,  S_t = S' + beta_t k_t u^T,
 * o_t = scale S_t^T q_t,  and D the gradient of the loss with respect to S_t
 * (coming from all later tokens), one token contributes, in this order:
 *
 *     D       += scale q_t do_t^T
 *     dq_t     = scale S_t do_t
 *     dbeta_t  = k_t^T D u
 *     du       = beta_t D^T k_t                 dv_t = du
 *     dk_t     = beta_t D u - S' du
 *     D'       = D - k_t du^T                   (gradient with respect to S')
 *     dlog_alpha_t[c] = sum_v D'[c,v] S'[c,v]   (S' = exp(log_alpha) . S_{t-1})
 *     D       <- Diag(alpha_t) D'               (gradient with respect to S_{t-1})
 *
 * The states S_{t-1} are needed in reverse order: the forward pass keeps one
 * state per block of kBwdBlock tokens and each block is replayed forward into a
 * buffer before it is walked backward.  Nothing is chunked in the arithmetic.
 * ---------------------------------------------------------------------------
 */
#define kBwdBlock 32

static void token_forward(const float *q, const float *k, const float *v, const float *log_alpha,
                          const float *beta, int64_t tok, int dk, int dv, double *S)
{
    (void)q;
    const double b = (double)beta[tok];
    for (int i = 0; i < dk; ++i) {
        const double a = exp((double)log_alpha[tok * dk + i]);
        for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] *= a;
    }
    double *u = (double *)malloc(sizeof(double) * (size_t)dv);
    for (int j = 0; j < dv; ++j) u[j] = 0.0;
    for (int i = 0; i < dk; ++i)
        for (int j = 0; j < dv; ++j) u[j] += (double)k[tok * dk + i] * S[(size_t)i * dv + j];
    for (int j = 0; j < dv; ++j) u[j] = (double)v[tok * dv + j] - u[j];
    for (int i = 0; i < dk; ++i)
        for (int j = 0; j < dv; ++j) S[(size_t)i * dv + j] += b * (double)k[tok * dk + i] * u[j];
    free(u);
}

/*
 * Gradients of  loss = sum(o . do) + sum(hT . dhT)  with respect to every input.
 *   do  : [B,T,H,dv] double          dhT : [N,H,dk,dv] double or NULL (zeros)
 *   dq,dk,dlog_alpha : [B,T,H,dk]    dv : [B,T,H,dv]    dbeta : [B,T,H]   (double, written;
 *   tokens that belong to no sequence get zeros)       dh0 : [N,H,dk,dv] double or NULL
 * Other arguments as in kda_oracle_forward.  Returns 0 on success.
 */
int kda_oracle_backward(int64_t B, int64_t T, int H, int dk, int dv, int64_t N,
                        const float *q, const float *k, const float *v,
                        const float *log_alpha, const float *beta,
                        const double *h0, const int64_t *cu_seqlens, double scale,
                        const double *d_o, const double *dhT,
                        double *dq, double *dk_out, double *dv_out, double *dla, double *dbeta,
                        double *dh0)
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
    const size_t ntok = (size_t)B * (size_t)T * (size_t)H;
    memset(dq, 0, sizeof(double) * ntok * dk);
    memset(dk_out, 0, sizeof(double) * ntok * dk);
    memset(dla, 0, sizeof(double) * ntok * dk);
    memset(dv_out, 0, sizeof(double) * ntok * dv);
    memset(dbeta, 0, sizeof(double) * ntok);

    const int64_t pairs = N * (int64_t)H;
    const size_t ssz = (size_t)dk * dv;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < pairs; ++p) {
        const int64_t n = p / H;
        const int h = (int)(p % H);
        int64_t row, t0, t1;
        if (cu_seqlens) { row = 0; t0 = cu_seqlens[n]; t1 = cu_seqlens[n + 1]; }
        else            { row = n; t0 = 0;             t1 = T; }
        const int64_t len = t1 - t0;
        const int64_t nblk = (len + kBwdBlock - 1) / kBwdBlock;

        /* forward: the state at the start of every block */
        double *ckpt = (double *)malloc(sizeof(double) * ssz * (size_t)(nblk + 1));
        double *S = (double *)malloc(sizeof(double) * ssz);
        if (h0) memcpy(S, h0 + (size_t)p * ssz, sizeof(double) * ssz);
        else    memset(S, 0, sizeof(double) * ssz);
        for (int64_t b = 0; b < nblk; ++b) {
            memcpy(ckpt + (size_t)b * ssz, S, sizeof(double) * ssz);
            const int64_t e = (b + 1) * kBwdBlock < len ? (b + 1) * kBwdBlock : len;
            for (int64_t t = b * kBwdBlock; t < e; ++t)
                token_forward(q, k, v, log_alpha, beta, (row * T + t0 + t) * H + h, dk, dv, S);
        }

        /* D = dL/dS_T */
        double *D = (double *)malloc(sizeof(double) * ssz);
        if (dhT) memcpy(D, dhT + (size_t)p * ssz, sizeof(double) * ssz);
        else     memset(D, 0, sizeof(double) * ssz);

        double *prev = (double *)malloc(sizeof(double) * ssz * kBwdBlock);   /* S_{t-1} per token */
        double *Sp = (double *)malloc(sizeof(double) * ssz);                 /* S' */
        double *u = (double *)malloc(sizeof(double) * (size_t)(2 * dv));
        double *du = u + dv;

        for (int64_t b = nblk - 1; b >= 0; --b) {
            const int64_t s = b * kBwdBlock;
            const int64_t e = s + kBwdBlock < len ? s + kBwdBlock : len;
            memcpy(S, ckpt + (size_t)b * ssz, sizeof(double) * ssz);
            for (int64_t t = s; t < e; ++t) {
                memcpy(prev + (size_t)(t - s) * ssz, S, sizeof(double) * ssz);
                token_forward(q, k, v, log_alpha, beta, (row * T + t0 + t) * H + h, dk, dv, S);
            }
            for (int64_t t = e - 1; t >= s; --t) {
                const int64_t tok = (row * T + t0 + t) * H + h;
                const double *Sm = prev + (size_t)(t - s) * ssz;
                const double bt = (double)beta[tok];
                /* replay the token: S', u, S_t (into S) */
                for (int i = 0; i < dk; ++i) {
                    const double a = exp((double)log_alpha[tok * dk + i]);
                    for (int j = 0; j < dv; ++j) Sp[(size_t)i * dv + j] = a * Sm[(size_t)i * dv + j];
                }
                for (int j = 0; j < dv; ++j) u[j] = 0.0;
                for (int i = 0; i < dk; ++i)
                    for (int j = 0; j < dv; ++j) u[j] += (double)k[tok * dk + i] * Sp[(size_t)i * dv + j];
                for (int j = 0; j < dv; ++j) u[j] = (double)v[tok * dv + j] - u[j];
                for (int i = 0; i < dk; ++i)
                    for (int j = 0; j < dv; ++j)
                        S[(size_t)i * dv + j] = Sp[(size_t)i * dv + j] + bt * (double)k[tok * dk + i] * u[j];

                /* D += scale q do^T ;  dq = scale S_t do */
                for (int i = 0; i < dk; ++i) {
                    double acc = 0.0;
                    for (int j = 0; j < dv; ++j) {
                        D[(size_t)i * dv + j] += scale * (double)q[tok * dk + i] * d_o[tok * dv + j];
                        acc += S[(size_t)i * dv + j] * d_o[tok * dv + j];
                    }
                    dq[tok * dk + i] = scale * acc;
                }
                /* dbeta = k^T D u ;  du = beta D^T k */
                double db = 0.0;
                for (int j = 0; j < dv; ++j) du[j] = 0.0;
                for (int i = 0; i < dk; ++i) {
                    const double ki = (double)k[tok * dk + i];
                    for (int j = 0; j < dv; ++j) {
                        db += ki * D[(size_t)i * dv + j] * u[j];
                        du[j] += ki * D[(size_t)i * dv + j];
                    }
                }
                for (int j = 0; j < dv; ++j) du[j] *= bt;
                dbeta[tok] = db;
                for (int j = 0; j < dv; ++j) dv_out[tok * dv + j] = du[j];
                /* dk = beta D u - S' du ;  D' = D - k du^T ;  dlog_alpha = rowsum(D' . S') ;
                   D <- Diag(alpha) D' */
                for (int i = 0; i < dk; ++i) {
                    const double ki = (double)k[tok * dk + i];
                    const double a = exp((double)log_alpha[tok * dk + i]);
                    double g1 = 0.0, g2 = 0.0, gl = 0.0;
                    for (int j = 0; j < dv; ++j) {
                        g1 += D[(size_t)i * dv + j] * u[j];
                        g2 += Sp[(size_t)i * dv + j] * du[j];
                        const double dprime = D[(size_t)i * dv + j] - ki * du[j];
                        gl += dprime * Sp[(size_t)i * dv + j];
                        D[(size_t)i * dv + j] = a * dprime;
                    }
                    dk_out[tok * dk + i] = bt * g1 - g2;
                    dla[tok * dk + i] = gl;
                }
            }
        }
        if (dh0) memcpy(dh0 + (size_t)p * ssz, D, sizeof(double) * ssz);
        free(u); free(Sp); free(prev); free(D); free(S); free(ckpt);
    }
    return 0;
}
