// Chunkwise KDA prefill in fp32 throughout (Section 3.1), in one kernel: what fp32 inputs get when the
// caller brings no workspace (with one, the parallel per-chunk kernel and the matrix-core walk of
// kda_chunk_bwd.hip run instead).
//
// One workgroup walks the chunks of one (sequence, head) for a 32-column slice
// of the state; every column of S is an independent recurrence, so slices never
// communicate.  Per chunk it evaluates, with plain fp32 FMAs on LDS tiles:
//
//   G        inclusive running sum of log2(alpha) inside the chunk
//   A_kk,A_qk[r,i] = sum_d x_r,d k_i,d 2^(G_r,d - G_i,d)   (pairwise, log domain,
//            so no 1/Gamma ever appears and nothing can overflow)
//   L = StrictTril(Diag(beta) A_kk),  X = (I + L)^-1 by forward substitution,
//   M = X Diag(beta)                                         (UT transform)
//   V_new = U - W S = M (V - (Gamma.K) S)                    ("pseudo"-value)
//   O = (Gamma.Q) S + Tril(A_qk) V_new
//   S <- Diag(gamma^C) S + (Gamma^{i->C}.K)^T V_new
//
// W and U are never materialised: U - W S = M V - M (Gamma.K) S, which saves two
// tiles of LDS and is the same arithmetic up to association.  Rows past the end
// of a short last chunk are padded with log_alpha = 0, beta = 0, k = q = v = 0,
// which are identity transitions.  This path is written for accuracy and
// clarity (it carries config-sized fp32 problems and serves as an on-GPU
// cross-check); the matrix-core path for bf16 inputs lives in kda_chunk_mfma.hip.
#include "kda_common.h"

namespace kda {

constexpr int kSimpleBV = 32;                       // state columns per workgroup
constexpr int kSimpleLdA = kChunk + 2;              // row stride of the packed A tile

template <int D> constexpr size_t simple_lds_floats()
{
    return 3 * kChunk * (D + 1) + kChunk * kSimpleLdA + 2 * kChunk * kSimpleBV + D * kSimpleBV
           + kChunk + D;
}

template <typename Tin, int D>
__global__ __launch_bounds__(256)
void kda_chunk_f32_kernel(const Tin *__restrict__ q, const Tin *__restrict__ k,
                          const Tin *__restrict__ v, const Tin *__restrict__ log_alpha,
                          const Tin *__restrict__ beta, const float *__restrict__ h0,
                          const int32_t *__restrict__ cu_seqlens, float *__restrict__ o,
                          float *__restrict__ hT, int64_t T, int H, float scale)
{
    constexpr int C = kChunk, LD = D + 1, LA = kSimpleLdA, BV = kSimpleBV;
    extern __shared__ float smem[];
    float *sQ = smem;                 // [C][LD]  q, later Gamma.Q
    float *sK = sQ + C * LD;          // [C][LD]  k, later Gamma^{i->C}.K
    float *sG = sK + C * LD;          // [C][LD]  log2 decay, its running sum, later Gamma.K
    float *sA = sG + C * LD;          // [C][LA]  strict lower: L -> X-I -> M (diag: beta);
                                      //          A_qk[r][i] is kept at [i][r+1] (upper part)
    float *sV = sA + C * LA;          // [C][BV]  V slice, later V - (Gamma.K) S
    float *sVn = sV + C * BV;         // [C][BV]  V_new
    float *sS = sVn + C * BV;         // [D][BV]  state slice
    float *sBeta = sS + D * BV;       // [C]
    float *sGend = sBeta + C;         // [D]      running sum at the last row of the chunk

    const int n = blockIdx.x, h = blockIdx.y, slice = blockIdx.z;
    const int tid = threadIdx.x;
    const int col0 = slice * BV;

    int64_t tok_base, len;
    if (cu_seqlens) { tok_base = cu_seqlens[n]; len = (int64_t)cu_seqlens[n + 1] - tok_base; }
    else            { tok_base = (int64_t)n * T; len = T; }

    const int64_t state_off = ((int64_t)n * H + h) * (int64_t)(D * D);
    for (int idx = tid; idx < D * BV; idx += 256) {
        const int d = idx / BV, c = idx % BV;
        sS[idx] = h0 ? h0[state_off + (int64_t)d * D + col0 + c] : 0.f;
    }

    for (int64_t c0 = 0; c0 < len; c0 += C) {
        const int nv = (int)((len - c0 < C) ? (len - c0) : C);
        const int64_t tok0 = tok_base + c0;

        // ---- load the chunk (zero padding past nv) ----
        for (int idx = tid; idx < C * D; idx += 256) {
            const int r = idx / D, d = idx % D;
            float fq = 0.f, fk = 0.f, fg = 0.f;
            if (r < nv) {
                const int64_t off = ((tok0 + r) * H + h) * (int64_t)D + d;
                fq = load_as_float(q + off);
                fk = load_as_float(k + off);
                fg = load_as_float(log_alpha + off) * kLog2e;
            }
            sQ[r * LD + d] = fq; sK[r * LD + d] = fk; sG[r * LD + d] = fg;
        }
        for (int idx = tid; idx < C * BV; idx += 256) {
            const int r = idx / BV, c = idx % BV;
            sV[idx] = (r < nv) ? load_as_float(v + ((tok0 + r) * H + h) * (int64_t)D + col0 + c) : 0.f;
        }
        if (tid < C) sBeta[tid] = (tid < nv) ? load_as_float(beta + (tok0 + tid) * H + h) : 0.f;
        __syncthreads();

        // ---- G: inclusive running sum of log2(alpha) over the chunk's tokens ----
        if (tid < D) {
            float run = 0.f;
            for (int r = 0; r < C; ++r) { run += sG[r * LD + tid]; sG[r * LD + tid] = run; }
            sGend[tid] = run;
        }
        __syncthreads();

        // ---- A_kk, A_qk for i <= r, pairwise in the log domain ----
        {
            const int i = tid & 63;
            for (int r = tid >> 6; r < C; r += 4) {
                if (i <= r) {
                    float akk = 0.f, aqk = 0.f;
                    for (int d = 0; d < D; ++d) {
                        const float e = fast_exp2(sG[r * LD + d] - sG[i * LD + d]);
                        const float t = sK[i * LD + d] * e;
                        akk = fmaf(sK[r * LD + d], t, akk);
                        aqk = fmaf(sQ[r * LD + d], t, aqk);
                    }
                    if (i < r) sA[r * LA + i] = sBeta[r] * akk;    // L = StrictTril(Diag(beta) A_kk)
                    sA[i * LA + r + 1] = aqk;                       // Tril(A_qk), stored transposed
                }
            }
        }
        __syncthreads();

        // ---- forward substitution: strict lower part becomes (I + L)^-1 - I ----
        for (int r = 1; r < C; ++r) {
            float val = 0.f;
            const int j = tid;
            if (j < r) {
                val = -sA[r * LA + j];
                for (int i = j + 1; i < r; ++i) val = fmaf(-sA[r * LA + i], sA[i * LA + j], val);
            }
            __syncthreads();
            if (j < r) sA[r * LA + j] = val;
            __syncthreads();
        }
        // M = X Diag(beta)
        for (int idx = tid; idx < C * C; idx += 256) {
            const int r = idx >> 6, j = idx & 63;
            if (j < r) sA[r * LA + j] *= sBeta[j];
            else if (j == r) sA[r * LA + j] = sBeta[j];
        }

        // ---- decay-scaled operands, in place ----
        for (int idx = tid; idx < C * D; idx += 256) {
            const int r = idx / D, d = idx % D;
            const float G = sG[r * LD + d];
            const float kk = sK[r * LD + d];
            const float gam = fast_exp2(G);
            sQ[r * LD + d] *= gam;                               // Gamma . Q
            sG[r * LD + d] = kk * gam;                           // Gamma . K
            sK[r * LD + d] = kk * fast_exp2(sGend[d] - G);       // Gamma^{i->C} . K
        }
        __syncthreads();

        // ---- sV <- V - (Gamma.K) S ----
        {
            const int c = tid & 31;
            for (int r = tid >> 5; r < C; r += 8) {
                float acc = 0.f;
                for (int d = 0; d < D; ++d) acc = fmaf(sG[r * LD + d], sS[d * BV + c], acc);
                sV[r * BV + c] -= acc;
            }
        }
        __syncthreads();

        // ---- V_new = M (V - (Gamma.K) S) ----
        {
            const int c = tid & 31;
            for (int r = tid >> 5; r < C; r += 8) {
                float acc = 0.f;
                for (int j = 0; j <= r; ++j) acc = fmaf(sA[r * LA + j], sV[j * BV + c], acc);
                sVn[r * BV + c] = acc;
            }
        }
        __syncthreads();

        // ---- O = (Gamma.Q) S + Tril(A_qk) V_new ----
        {
            const int c = tid & 31;
            for (int r = tid >> 5; r < nv; r += 8) {
                float acc = 0.f;
                for (int d = 0; d < D; ++d) acc = fmaf(sQ[r * LD + d], sS[d * BV + c], acc);
                for (int i = 0; i <= r; ++i) acc = fmaf(sA[i * LA + r + 1], sVn[i * BV + c], acc);
                o[((tok0 + r) * H + h) * (int64_t)D + col0 + c] = acc * scale;
            }
        }
        __syncthreads();

        // ---- S <- Diag(gamma^C) S + (Gamma^{i->C}.K)^T V_new ----
        {
            const int c = tid & 31;
            for (int d = tid >> 5; d < D; d += 8) {
                float acc = sS[d * BV + c] * fast_exp2(sGend[d]);
                for (int j = 0; j < C; ++j) acc = fmaf(sK[j * LD + d], sVn[j * BV + c], acc);
                sS[d * BV + c] = acc;
            }
        }
        __syncthreads();
    }

    if (hT) {
        __syncthreads();
        for (int idx = tid; idx < D * BV; idx += 256) {
            const int d = idx / BV, c = idx % BV;
            hT[state_off + (int64_t)d * D + col0 + c] = sS[idx];
        }
    }
}

template <typename Tin, int D>
static kda_status launch_chunk_f32(const kda_dims *dm, const void *q, const void *k, const void *v,
                                   const void *log_alpha, const void *beta, const float *h0,
                                   const int32_t *cu, void *o, float *hT, hipStream_t stream)
{
    auto kern = kda_chunk_f32_kernel<Tin, D>;
    const size_t lds = simple_lds_floats<D>() * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess)
        return fail(KDA_ERR_LAUNCH, "kda_chunk_f32_kernel: cannot reserve %zu B of LDS: %s", lds,
                    hipGetErrorString(e));
    if (dm->num_seqs == 0 || dm->heads == 0) return KDA_OK;
    dim3 grid((unsigned)dm->num_seqs, (unsigned)dm->heads, (unsigned)(D / kSimpleBV));
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream,
                       static_cast<const Tin *>(q), static_cast<const Tin *>(k),
                       static_cast<const Tin *>(v), static_cast<const Tin *>(log_alpha),
                       static_cast<const Tin *>(beta), h0, cu, static_cast<float *>(o), hT,
                       (int64_t)dm->seqlen, (int)dm->heads, dm->scale);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_chunk_f32_kernel: %s", hipGetErrorString(e));
    return KDA_OK;
}

kda_status chunk_f32_dispatch(const kda_dims *dm, const void *q, const void *k, const void *v,
                              const void *log_alpha, const void *beta, const float *h0,
                              const int32_t *cu, void *o, float *hT, hipStream_t stream)
{
    const bool bf = dm->in_dtype == KDA_BF16;
    if (dm->dk == 128)
        return bf ? launch_chunk_f32<__hip_bfloat16, 128>(dm, q, k, v, log_alpha, beta, h0, cu, o, hT, stream)
                  : launch_chunk_f32<float, 128>(dm, q, k, v, log_alpha, beta, h0, cu, o, hT, stream);
    return bf ? launch_chunk_f32<__hip_bfloat16, 64>(dm, q, k, v, log_alpha, beta, h0, cu, o, hT, stream)
              : launch_chunk_f32<float, 64>(dm, q, k, v, log_alpha, beta, h0, cu, o, hT, stream);
}

}  // namespace kda
