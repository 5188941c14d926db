// Chunkwise backward pass of KDA in fp32 (gradients of Section 3, Eq. (1) through the chunkwise
// form of Section 3.1).  The paper derives no backward algorithm; this one is the chain rule
// applied to the chunk equations, with every decay kept as a pairwise difference in the log
// domain (2^(G_r - G_i) with i <= r, 2^(G_r), 2^(G_C - G_r): all at most 1), so that nothing
// can overflow whatever the decay.
//
// Per chunk of C = 64 tokens (G inclusive running sum of log alpha, S0 the state at the chunk's
// start, beta, k, q, v the chunk's rows):
//
//   forward    A_kk[r,i] = sum_d k_r,d k_i,d e^(G_r,d - G_i,d),  A_qk likewise with q_r
//              L = StrictTril(Diag(beta) A_kk),  T = (I + L)^-1,  M = T Diag(beta)
//              Kg = Gamma.K,  Qg = Gamma.Q,  Kt = Gamma^{i->C}.K,  P = Tril(A_qk)
//              Y = V - Kg S0,   Vn = M Y                               ("pseudo"-values)
//              O = scale (Qg S0 + P Vn),   S1 = Diag(e^(G_C)) S0 + Kt^T Vn
//
//   backward   (dO pre-multiplied by scale, dS1 the gradient of the chunk's end state)
//              dVn = P^T dO + Kt dS1            X = M^T dVn   (= dV)
//              dS0 = Diag(e^(G_C)) dS1 + Qg^T dO - Kg^T X
//              dQg = dO S0^T    dKg = -X S0^T    dKt = Vn dS1^T
//              dP  = Tril(dO Vn^T)               dM  = Tril(dVn Y^T)
//              dT  = dM Diag(beta)               dbeta_j  = sum_r dM[r,j] T[r,j]
//              dL  = -StrictTril(T^T dT T^T)     dbeta_r += sum_i dL[r,i] A_kk[r,i]
//              dA_kk = Diag(beta) dL
//              dq_r = Gamma_r . dQg_r + sum_{i<=r} dP[r,i] k_i e^(G_r - G_i)
//              dk_t = Gamma_t . dKg_t + e^(G_C - G_t) . dKt_t
//                     + sum_{i<t} dA_kk[t,i] k_i e^(G_t - G_i)
//                     + sum_{r>t} dA_kk[r,t] k_r e^(G_r - G_t) + sum_{r>=t} dP[r,t] q_r e^(G_r - G_t)
//              dG_t = (every product above that carries e^(+G_t)) - (those that carry e^(-G_t)),
//              dG_C = e^(G_C) . rowsum(dS1 . S0) + sum_t dKt_t . Kt_t
//              dlog_alpha_t = sum_{r>=t} dG_r + dG_C
//
// Decays that cross a 16-token block are split at the end E of the earlier block,
// e^(G_r - G_i) = e^(G_r - E) e^(E - G_i) (both factors at most 1 whatever the decay), which turns those
// parts of A_kk, A_qk and of the gradient sums into block products of decay-scaled operands; only
// inside a 16 x 16 diagonal block is there one exponential per pair and channel.
//
// Five kernels in fp32, 512 threads each (LDS leaves room for one workgroup per compute unit); every
// dense product runs on the matrix cores with fp32 operands (v_mfma_f32_16x16x4_f32,
// v_mfma_f32_32x32x2_f32):
//   kda_bwd_prep     one workgroup per (chunk, head), all chunks in parallel: A_kk, A_qk, T and M,
//                    left in the workspace as two packed C x C tiles, and the decay-scaled operands
//                    Gamma.Q, Gamma.K, Gamma^{i->C}.K for the two scans
//   kda_bwd_states   one workgroup per (sequence, head, 32 state columns) walks the chunks
//                    forward and leaves S0 of every chunk, Y and Vn in the workspace
//   kda_bwd_scan     the same decomposition walks the chunks backward with dS: dVn, dV, the dS1
//                    of every chunk, dh0  (the columns of S never mix, neither do those of dS)
//   kda_bwd_products one workgroup per (chunk, head): the products with S0 and dS1 (dQg, dKg,
//                    dKt, dG_C) folded into dq, dk and dG, and the two C x C products dP, dM
//   kda_bwd_chain    one workgroup per (chunk, head): the gradient through T and the decay terms
//                    of dq, dk, dG, the reverse running sum that turns dG into dlog_alpha, dbeta
#include "kda_common.h"

namespace kda {
namespace {

constexpr int kC = kChunk;
constexpr int kBV = 32;                 // state columns per workgroup of the two scans
constexpr int kLA = kC + 2;             // row stride of a packed C x C tile
constexpr int kTile = kC * kLA;         // floats in one
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Slot of chunk c of sequence n among all chunk slots (times H + h gives the workspace index).
// Packed batches: floor(cu[n] / C) + n + c is strictly increasing over (n, c) and bounded by
// floor(total / C) + N.
__device__ __forceinline__ int64_t chunk_slot(const int32_t *cu, int n, int64_t chunks_per_seq, int64_t c)
{
    return cu ? (int64_t)(cu[n] / kC) + n + c : (int64_t)n * chunks_per_seq + c;
}

// ---- global -> LDS copies.  Every copy issues all of a thread's 16-byte loads before it touches
// LDS, so that their latencies overlap (a load-store-load-store loop pays one memory round trip
// per iteration).

__device__ __forceinline__ void unpack16(const uint4 &w, const float *, float (&f)[4])
{
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
}
__device__ __forceinline__ void unpack16(const uint4 &w, const __hip_bfloat16 *, float (&f)[8])
{
    unpack_bf16x2(w.x, f[0], f[1]); unpack_bf16x2(w.y, f[2], f[3]);
    unpack_bf16x2(w.z, f[4], f[5]); unpack_bf16x2(w.w, f[6], f[7]);
}

// ROWS x W block of Tin (rows `stride` elements apart, 16-byte aligned): fetch() issues the loads
// (rows r >= nv read as zero), commit() writes dst[r * ld + c] = mul * x.  ROWS * W * sizeof(Tin) / 16
// must be a multiple of the NT threads that take part (or less than NT).  Keeping the two apart lets a loop fetch its next
// block before it works on the current one.
template <typename Tin, int ROWS, int W, int NT = 256>
struct RowsFetch {
    static constexpr int EPV = 16 / (int)sizeof(Tin), VPR = W / EPV, TOTAL = ROWS * VPR, NV = (TOTAL + NT - 1) / NT;
    static_assert(TOTAL % NT == 0 || TOTAL < NT, "block size");
    uint4 buf[NV];
    __device__ __forceinline__ void fetch(const Tin *__restrict__ src, int64_t stride, int nv, int tid)
    {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int vi = tid + NT * u, r = vi / VPR, cv = vi % VPR;
            buf[u] = make_uint4(0u, 0u, 0u, 0u);
            if (vi < TOTAL && r < nv) buf[u] = *reinterpret_cast<const uint4 *>(src + r * stride + cv * EPV);
        }
    }
    __device__ __forceinline__ void commit(float *dst, int ld, float mul, int tid) const
    {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int vi = tid + NT * u, r = vi / VPR, cv = vi % VPR;
            float f[EPV];
            unpack16(buf[u], (const Tin *)nullptr, f);
            if (vi < TOTAL) {
                float *p = dst + r * ld + cv * EPV;
                if ((ld & 3) == 0) {                     // rows 16-byte aligned: whole 16-byte stores (dst is)
#pragma unroll
                    for (int e = 0; e < EPV; e += 4)
                        *reinterpret_cast<float4 *>(p + e) = make_float4(mul * f[e], mul * f[e + 1], mul * f[e + 2], mul * f[e + 3]);
                } else {
#pragma unroll
                    for (int e = 0; e < EPV; ++e) p[e] = mul * f[e];
                }
            }
        }
    }
};

template <typename Tin, int ROWS, int W, int NT = 256>
__device__ __forceinline__ void rows_to_lds(float *dst, int ld, const Tin *__restrict__ src, int64_t stride,
                                            int nv, float mul, int tid)
{
    RowsFetch<Tin, ROWS, W, NT> f;
    f.fetch(src, stride, nv, tid);
    f.commit(dst, ld, mul, tid);
}

// N4 contiguous 16-byte words, global -> LDS (both 16-byte aligned).
template <int N4, int NT = 256>
struct BlockFetch {
    static constexpr int NV = (N4 + NT - 1) / NT;
    uint4 buf[NV];
    __device__ __forceinline__ void fetch(const float *__restrict__ src, int tid)
    {
#pragma unroll
        for (int u = 0; u < NV; ++u)
            if (tid + NT * u < N4) buf[u] = reinterpret_cast<const uint4 *>(src)[tid + NT * u];
    }
    __device__ __forceinline__ void commit(float *dst, int tid) const
    {
#pragma unroll
        for (int u = 0; u < NV; ++u)
            if (tid + NT * u < N4) reinterpret_cast<uint4 *>(dst)[tid + NT * u] = buf[u];
    }
};

template <int N4>
__device__ __forceinline__ void copy_to_lds(float *dst, const float *__restrict__ src, int tid)
{
    BlockFetch<N4> f;
    f.fetch(src, tid);
    f.commit(dst, tid);
}

// In place: sG[r][d] <- sum over rows <= r, all NT threads (NT / D row groups per channel, prefix
// in registers, the groups' totals through sTot [NT / D][D]); sGend[d] = last row.  Ends with a barrier;
// the caller has one before.
template <int D, int NT = 256>
__device__ __forceinline__ void cumsum_rows(float *sG, float *sTot, float *sGend, int tid)
{
    constexpr int LD = D + 1, RG = NT / D, RPT = kC / RG;
    const int d = tid % D, rg = tid / D;
    float g[RPT];
#pragma unroll
    for (int u = 0; u < RPT; ++u) g[u] = sG[(rg * RPT + u) * LD + d];
#pragma unroll
    for (int u = 1; u < RPT; ++u) g[u] += g[u - 1];
    sTot[rg * D + d] = g[RPT - 1];
    __syncthreads();
    float off = 0.f;
    for (int r2 = 0; r2 < rg; ++r2) off += sTot[r2 * D + d];
#pragma unroll
    for (int u = 0; u < RPT; ++u) sG[(rg * RPT + u) * LD + d] = g[u] + off;
    if (rg == RG - 1) sGend[d] = g[RPT - 1] + off;
    __syncthreads();
}

// How the waves of a scan share a step's result tiles.  Products with token rows (64 x 32 results: four
// row tiles, two column tiles): with four waves a wave takes a row tile and both columns, with eight one
// tile.  Products with state rows (D x 32): D / 16 row tiles; a wave takes whole row tiles with both
// columns when there are enough of them, else one tile.
constexpr int kScanThreads = 512;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kTokCols = kScanWaves == 4 ? 2 : 1;
template <int D> struct StateTiles {
    static constexpr int NRT = D / 16;
    static constexpr bool kPair = NRT >= kScanWaves;
    static constexpr int NC = kPair ? 2 : 1, RPW = kPair ? NRT / kScanWaves : 1;
};

// The decay-scaled operands of a chunk as kda_bwd_prep leaves them in the workspace: three [C][D] fp32
// tiles (Gamma.Q, Gamma.K, Gamma^{i->C}.K; rows past the chunk's end are zero) and G_C in log2 units.
template <int D> constexpr int operand_floats() { return 3 * kC * D + D; }

// Everything a scan step reads from global memory, held in registers between fetch() and commit().
template <typename Tslice, int D, bool kWithQ>
struct StepFetch {
    RowsFetch<float, kC, D, kScanThreads> fq, fkg, fkt;
    RowsFetch<Tslice, kC, kBV, kScanThreads> fs;
    BlockFetch<kTile / 4, kScanThreads> ft;
    float gend;
    __device__ __forceinline__ void fetch(const float *ops, const Tslice *slice, const float *tile,
                                          int64_t tok0, int nv, int H, int h, int col0, int tid)
    {
        ft.fetch(tile, tid);
        if (kWithQ) fq.fetch(ops, D, kC, tid);
        fkg.fetch(ops + kC * D, D, kC, tid);
        fkt.fetch(ops + 2 * kC * D, D, kC, tid);
        fs.fetch(slice + (tok0 * H + h) * (int64_t)D + col0, (int64_t)H * D, nv, tid);
        gend = ops[3 * kC * D + tid % D];
    }
    // sQ <- Gamma.Q (if fetched), sG <- Gamma.K, sK <- Gamma^{i->C}.K, sA <- the M | A_qk tile
    __device__ __forceinline__ void commit(float *sQ, float *sK, float *sG, float *sA, float *sSlice,
                                           float *sGend, float slice_mul, int tid) const
    {
        constexpr int LD = D + 4;           // as in the scan kernels
        ft.commit(sA, tid);
        if (kWithQ) fq.commit(sQ, LD, 1.f, tid);
        fkg.commit(sG, LD, 1.f, tid);
        fkt.commit(sK, LD, 1.f, tid);
        fs.commit(sSlice, kBV, slice_mul, tid);
        if (tid < D) sGend[tid] = gend;
    }
};

// 16 x 16 fp32 matrix-core tile (v_mfma_f32_16x16x4_f32): with m = lane % 16 and g = lane / 16 a lane
// feeds A[m][k + g] and B[k + g][m] for every step k of four, and holds D[4 g + j][m] in register j.
// a(k) and b(k) return this lane's operand element for contraction index k (k + g already applied).
// kend - kbeg is a multiple of 8 everywhere (block boundaries): two steps per iteration, operands first.
template <typename FA, typename FB>
__device__ __forceinline__ f32x4 mma16(int kbeg, int kend, int g, f32x4 acc, FA &&a, FB &&b)
{
    for (int k = kbeg + g; k < kend; k += 8) {
        const float a0 = a(k), b0 = b(k), a1 = a(k + 4), b1 = b(k + 4);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc, 0, 0, 0);
    }
    return acc;
}

// NCT result tiles that share the A operand (one or both 16-column halves of a 32-column slice):
// acc[c] += A B_c with b(k, c).
template <int NCT, typename FA, typename FB>
__device__ __forceinline__ void mma16t(int kbeg, int kend, int g, f32x4 (&acc)[NCT], FA &&a, FB &&b)
{
    for (int k = kbeg + g; k < kend; k += 8) {
        const float a0 = a(k), a1 = a(k + 4);
        float b0[NCT], b1[NCT];
#pragma unroll
        for (int c = 0; c < NCT; ++c) { b0[c] = b(k, c); b1[c] = b(k + 4, c); }
#pragma unroll
        for (int c = 0; c < NCT; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0[c], acc[c], 0, 0, 0);
#pragma unroll
        for (int c = 0; c < NCT; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1[c], acc[c], 0, 0, 0);
    }
}

// Loads one chunk.  On return (the last statement is a barrier):
//   sQ, sK [C][D+1]  q and k as given (zero rows past nv)
//   sG     [C][D+1]  G in log2 units (rows past nv repeat the last valid row)
//   sBeta [C] (zero past nv), sGend [D] (G of the last row); sTot [NT] is scratch
template <typename Tin, int D, int NT = 256>
__device__ void chunk_load(const Tin *__restrict__ q, const Tin *__restrict__ k,
                           const Tin *__restrict__ log_alpha, const Tin *__restrict__ beta,
                           int64_t tok0, int nv, int H, int h, float *sQ, float *sK, float *sG,
                           float *sBeta, float *sGend, float *sTot, int tid)
{
    constexpr int LD = D + 1;
    const int64_t base = (tok0 * H + h) * (int64_t)D, stride = (int64_t)H * D;
    rows_to_lds<Tin, kC, D, NT>(sQ, LD, q + base, stride, nv, 1.f, tid);
    rows_to_lds<Tin, kC, D, NT>(sK, LD, k + base, stride, nv, 1.f, tid);
    rows_to_lds<Tin, kC, D, NT>(sG, LD, log_alpha + base, stride, nv, kLog2e, tid);
    if (tid < kC) sBeta[tid] = (tid < nv) ? load_as_float(beta + (tok0 + tid) * H + h) : 0.f;
    __syncthreads();
    cumsum_rows<D, NT>(sG, sTot, sGend, tid);
}

// q, k, G tiles -> Gamma.Q, Gamma^{i->C}.K, Gamma.K (in sQ, sK, sG), as the forward kernel does.
template <int D, int NT = 256>
__device__ void decay_operands(float *sQ, float *sK, float *sG, const float *sGend, int tid)
{
    constexpr int LD = D + 1;
    for (int idx = tid; idx < kC * D; idx += NT) {
        const int r = idx / D, d = idx % D;
        const float G = sG[r * LD + d];
        const float kk = sK[r * LD + d];
        const float gam = fast_exp2(G);
        sQ[r * LD + d] *= gam;
        sG[r * LD + d] = kk * gam;
        sK[r * LD + d] = kk * fast_exp2(sGend[d] - G);
    }
}

// The two packed C x C tiles of a chunk, [C][kLA] floats each, that kda_bwd_prep leaves in the
// workspace:
//   tile 0   strict lower part [r][i]: T - I          upper part [i][r+1], i <= r: A_kk[r][i]
//   tile 1   lower part with diagonal [r][j]: M = T Diag(beta)    upper part [i][r+1]: A_qk[r][i]

template <int NT = 256>
__device__ __forceinline__ void load_tile(float *dst, const float *__restrict__ src, int tid)
{
    BlockFetch<kTile / 4, NT> f;
    f.fetch(src, tid);
    f.commit(dst, tid);
}

constexpr int kPrepThreads = 1024;

template <typename Tin, int D>
__global__ __launch_bounds__(kPrepThreads)
void kda_bwd_prep_kernel(const Tin *__restrict__ q, const Tin *__restrict__ k,
                         const Tin *__restrict__ log_alpha, const Tin *__restrict__ beta,
                         const int32_t *__restrict__ cu, float *__restrict__ Tw, float *__restrict__ Ow,
                         int64_t T, int H, int64_t chunks_per_seq)
{
    constexpr int LD = D + 1, NT = kPrepThreads, NW = NT / 64;
    extern __shared__ float smem[];
    float *sQ = smem, *sK = sQ + kC * LD, *sG = sK + kC * LD;
    float *s0 = sG + kC * LD, *s1 = s0 + kTile;
    float *sBeta = s1 + kTile, *sGend = sBeta + kC, *sTot = sGend + D;

    const int64_t ci = blockIdx.y;
    const int n = blockIdx.x, h = blockIdx.z, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t c0 = ci * kC;
    if (c0 >= len) return;
    const int nv = (int)((len - c0 < kC) ? (len - c0) : kC);
    const int64_t slot = chunk_slot(cu, n, chunks_per_seq, ci) * H + h;

    for (int idx = tid; idx < 2 * kTile; idx += NT) s0[idx] = 0.f;
    chunk_load<Tin, D, NT>(q, k, log_alpha, beta, tok_base + c0, nv, H, h, sQ, sK, sG, sBeta, sGend, sTot, tid);
    auto put = [&](int r, int i, float akk, float aqk) {         // one entry with i <= r into both tiles
        if (i < r) {                                             // L = StrictTril(Diag(beta) A_kk), kept twice:
            s0[r * kLA + i] = sBeta[r] * akk;                    // s0 becomes T - I block by block,
            s1[r * kLA + i] = sBeta[r] * akk;                    // s1 keeps L until M replaces it
        }
        s0[i * kLA + r + 1] = akk;
        s1[i * kLA + r + 1] = aqk;
    };
    // A_kk, A_qk in 16-token blocks.  Below the diagonal (row block R > column block I) the decay splits at
    // the end of block I, E_I = G of its last token:  e^(G_r - G_i) = e^(G_r - E_I) e^(E_I - G_i), both
    // factors at most 1, so the block is a plain product of two decay-scaled operands: matrix cores,
    // one exponential per operand element.  Wave w takes the block pairs w, w + NT / 64, ... of the list below.
    {
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        for (int pair = wave; pair < 6; pair += NW) {
            const int R = pair < 3 ? pair + 1 : (pair < 5 ? pair - 1 : 3);        // (1,0) (2,0) (3,0) (2,1) (3,1) (3,2)
            const int I = pair < 3 ? 0 : (pair < 5 ? 1 : 2);
            const float *gE = sG + (16 * I + 15) * LD;
            const float *gr = sG + (16 * R + m) * LD, *gi = sG + (16 * I + m) * LD;
            const float *kr = sK + (16 * R + m) * LD, *qr = sQ + (16 * R + m) * LD, *ki = sK + (16 * I + m) * LD;
            f32x4 akk = {0.f, 0.f, 0.f, 0.f}, aqk = {0.f, 0.f, 0.f, 0.f};
            for (int d = g; d < D; d += 4) {
                const float e = gE[d];
                const float f = fast_exp2(gr[d] - e), b_ = ki[d] * fast_exp2(e - gi[d]);
                akk = __builtin_amdgcn_mfma_f32_16x16x4f32(kr[d] * f, b_, akk, 0, 0, 0);
                aqk = __builtin_amdgcn_mfma_f32_16x16x4f32(qr[d] * f, b_, aqk, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) put(16 * R + 4 * g + j, 16 * I + m, akk[j], aqk[j]);
        }
    }
    // The four diagonal blocks pair by pair in the log domain (the decay inside a block may exceed any
    // factorisation's range): 256 threads (r, i) per set of blocks, NT / 256 sets side by side.
    {
        constexpr int kSets = NT / 256, kPer = 4 / kSets;
        const int rl = (tid & 255) >> 4, il = tid & 15, first = kPer * (tid >> 8);
        float akk[kPer] = {}, aqk[kPer] = {};
        for (int d = 0; d < D; ++d) {
#pragma unroll
            for (int b4 = 0; b4 < kPer; ++b4) {
                const int r = 16 * (first + b4) + rl, i = 16 * (first + b4) + il;
                const float t = sK[i * LD + d] * fast_exp2(fminf(sG[r * LD + d] - sG[i * LD + d], 0.f));
                akk[b4] = fmaf(sK[r * LD + d], t, akk[b4]);
                aqk[b4] = fmaf(sQ[r * LD + d], t, aqk[b4]);
            }
        }
#pragma unroll
        for (int b4 = 0; b4 < kPer; ++b4)
            if (il <= rl) put(16 * (first + b4) + rl, 16 * (first + b4) + il, akk[b4], aqk[b4]);
    }
    __syncthreads();
    // (I + L)^-1 - I in 16 x 16 blocks.  Diagonal blocks: wave w inverts block w, lane m < 16 its column m
    // (X[r][m] = -L[r][m] - sum_{m < i < r} L[r][i] X[i][m]; a lane reads back only what it wrote itself).
    {
        const int wave = tid >> 6, lane = tid & 63, b0 = 16 * wave;
        if (wave < 4 && lane < 16) {
            for (int r = 1; r < 16; ++r) {
                float val = 0.f;
                if (lane < r) {
                    val = -s1[(b0 + r) * kLA + b0 + lane];
                    for (int i = lane + 1; i < r; ++i)
                        val = fmaf(-s1[(b0 + r) * kLA + b0 + i], s0[(b0 + i) * kLA + b0 + lane], val);
                    s0[(b0 + r) * kLA + b0 + lane] = val;
                }
            }
        }
    }
    __syncthreads();
    // Blocks below the diagonal, one block row at a time (block (R, I) needs the blocks (J, I), I <= J < R):
    // X_RI = -X_RR (sum_J L_RJ X_JI), X_RR and X_II with their unit diagonals; wave I takes column block I.
    {
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        auto X = [&](int r, int c) { return r == c ? 1.f : (c < r ? s0[r * kLA + c] : 0.f); };
        for (int R = 1; R < 4; ++R) {
            if (wave < R) {
                const int I = wave;
                const f32x4 t = mma16(16 * I, 16 * R, g, f32x4{0.f, 0.f, 0.f, 0.f},
                                      [&](int k) { return s1[(16 * R + m) * kLA + k]; },          // L[16 R + m][k]
                                      [&](int k) { return X(k, 16 * I + m); });
                // the second product's B operand B[k][m] = t(k, m) sits in register k % 4 of lane group
                // k / 4: with contraction slot (step ks, group g) standing for k = 4 g + ks, register ks
                // of this lane is its operand as it stands
                f32x4 r = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    r = __builtin_amdgcn_mfma_f32_16x16x4f32(X(16 * R + m, 16 * R + 4 * g + ks), t[ks], r, 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j) s0[(16 * R + 4 * g + j) * kLA + 16 * I + m] = -r[j];
            }
            __syncthreads();
        }
    }
    for (int idx = tid; idx < kC * kC; idx += NT) {
        const int r = idx >> 6, j = idx & 63;
        if (j < r) s1[r * kLA + j] = s0[r * kLA + j] * sBeta[j];
        else if (j == r) s1[r * kLA + j] = sBeta[j];
    }
    __syncthreads();
    float *dst = Tw + slot * (int64_t)(2 * kTile);
    for (int idx = tid; idx < 2 * kTile; idx += NT) dst[idx] = s0[idx];
    // the decay-scaled operands for the two scans
    decay_operands<D, NT>(sQ, sK, sG, sGend, tid);                  // sQ <- Gamma.Q, sG <- Gamma.K, sK <- Gamma^{i->C}.K
    __syncthreads();
    float *ops = Ow + slot * (int64_t)operand_floats<D>();
    for (int idx = tid; idx < kC * D / 4; idx += NT) {
        const int r = idx / (D / 4), c = 4 * (idx % (D / 4));
        const float *pq = sQ + r * LD + c, *pg = sG + r * LD + c, *pk = sK + r * LD + c;
        reinterpret_cast<float4 *>(ops)[idx] = make_float4(pq[0], pq[1], pq[2], pq[3]);
        reinterpret_cast<float4 *>(ops + kC * D)[idx] = make_float4(pg[0], pg[1], pg[2], pg[3]);
        reinterpret_cast<float4 *>(ops + 2 * kC * D)[idx] = make_float4(pk[0], pk[1], pk[2], pk[3]);
    }
    if (tid < D) ops[3 * kC * D + tid] = sGend[tid];
}

template <int D> constexpr size_t prep_lds_floats() { return 3 * kC * (D + 1) + 2 * kTile + kC + D + kPrepThreads; }

template <int D> constexpr size_t scan_lds_floats()          // kda_bwd_scan
{
    return 3 * kC * (D + 4) + kC * kLA + 3 * kC * kBV + D * kBV + D;
}

template <int D> constexpr size_t states_lds_floats()        // kda_bwd_states
{
    return 2 * kC * (D + 4) + kC * kLA + 2 * kC * kBV + D * kBV + D;
}

// ------------------------------------------------------------------------------------------
// Forward walk: S0 of every chunk, Y = V - Kg S0 and Vn = M Y.
// ------------------------------------------------------------------------------------------
template <typename Tin, int D>
__global__ __launch_bounds__(kScanThreads)
void kda_bwd_states_kernel(const Tin *__restrict__ v, const float *__restrict__ h0,
                           const int32_t *__restrict__ cu, const float *__restrict__ Tw,
                           const float *__restrict__ Ow,
                           float *__restrict__ Sc, float *__restrict__ Yw, float *__restrict__ Vnw,
                           int64_t T, int H,
                           int64_t chunks_per_seq)
{
    constexpr int LD = D + 4;          // rows 16-byte aligned: the operand tiles are written 16 bytes at a time
    extern __shared__ float smem[];
    float *sK = smem, *sG = sK + kC * LD, *sA = sG + kC * LD;        // Gamma^{i->C}.K, Gamma.K, M | A_qk
    float *sV = sA + kC * kLA, *sVn = sV + kC * kBV;                 // V slice -> Y, V_new
    float *sS = sVn + kC * kBV, *sGend = sS + D * kBV;               // state slice, G_C

    const int n = blockIdx.x, h = blockIdx.y, col0 = blockIdx.z * kBV, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t state_off = ((int64_t)n * H + h) * (int64_t)(D * D);
    for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
        const int d = idx / kBV, c = idx % kBV;
        sS[idx] = h0 ? h0[state_off + (int64_t)d * D + col0 + c] : 0.f;
    }

    const int64_t nchunks = (len + kC - 1) / kC;
    const int64_t slot_first = chunk_slot(cu, n, chunks_per_seq, 0) * H + h;     // slots of a sequence are H apart
    auto valid_rows = [&](int64_t ci) { return (int)((len - ci * kC < kC) ? (len - ci * kC) : kC); };
    StepFetch<Tin, D, false> nxt;
    if (nchunks > 0)
        nxt.fetch(Ow + slot_first * (int64_t)operand_floats<D>(), v, Tw + (slot_first * 2 + 1) * (int64_t)kTile,
                  tok_base, valid_rows(0), H, h, col0, tid);
    for (int64_t ci = 0; ci < nchunks; ++ci) {
        const int nv = valid_rows(ci);
        const int64_t tok0 = tok_base + ci * kC;
        const int64_t slot = slot_first + ci * H;
        __syncthreads();
        for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
            const int d = idx / kBV, c = idx % kBV;
            Sc[slot * (int64_t)(D * D) + (int64_t)d * D + col0 + c] = sS[idx];
        }
        nxt.commit(nullptr, sK, sG, sA, sV, sGend, 1.f, tid);
        if (ci + 1 < nchunks)                                    // the next chunk's loads fly during this one's work
            nxt.fetch(Ow + (slot + H) * (int64_t)operand_floats<D>(), v, Tw + ((slot + H) * 2 + 1) * (int64_t)kTile,
                      tok0 + kC, valid_rows(ci + 1), H, h, col0, tid);
        __syncthreads();
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        const int r0 = 16 * (wave & 3);                          // this wave's 16 token rows ...
        const int cb = kTokCols == 2 ? 0 : 16 * (wave >> 2);     // ... and first slice column
        f32x4 y[kTokCols] = {};
        mma16t<kTokCols>(0, D, g, y, [&](int k) { return sG[(r0 + m) * LD + k]; },                    // Kg S0
                         [&](int k, int c) { return sS[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)                       // Y = V - Kg S0
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                y[c][j] = sV[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] - y[c][j];
                sV[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = y[c][j];
            }
        __syncthreads();
        f32x4 vn[kTokCols] = {};
        mma16t<kTokCols>(0, r0 + 16, g, vn, [&](int k) { return k <= r0 + m ? sA[(r0 + m) * kLA + k] : 0.f; },   // Vn = M Y
                         [&](int k, int c) { return sV[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) sVn[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = vn[c][j];
        __syncthreads();
        for (int idx = tid; idx < nv * kBV; idx += kScanThreads) {       // whole 128-byte rows of the slice at a time
            const int64_t off = ((tok0 + idx / kBV) * H + h) * (int64_t)D + col0 + idx % kBV;
            Yw[off] = sV[idx];
            Vnw[off] = sVn[idx];
        }
        using ST = StateTiles<D>;
        for (int q = 0; q < ST::RPW; ++q) {                              // S1 = Diag(e^G_C) S0 + Kt^T Vn
            const int d0 = 16 * (ST::kPair ? wave * ST::RPW + q : wave % ST::NRT);
            const int sb = ST::kPair ? 0 : 16 * (wave / ST::NRT);
            f32x4 acc[ST::NC];
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[c][j] = sS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] * fast_exp2(sGend[d0 + 4 * g + j]);
            mma16t<ST::NC>(0, kC, g, acc, [&](int k) { return sK[k * LD + d0 + m]; },
                           [&](int k, int c) { return sVn[k * kBV + sb + 16 * c + m]; });
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j) sS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] = acc[c][j];
        }
    }
}

// ------------------------------------------------------------------------------------------
// The forward pass itself from the same pieces (fp32 inputs, or bf16 inputs when the fp32 path is
// asked for): kda_bwd_prep, then this walk, which is kda_bwd_states plus
// O = scale (Qg S0 + P Vn) and keeps nothing but o and the final state.
// ------------------------------------------------------------------------------------------
template <int D> constexpr size_t fwd_scan_lds_floats()
{
    return 3 * kC * (D + 4) + kC * kLA + 2 * kC * kBV + D * kBV + D;
}

template <typename Tin, int D>
__global__ __launch_bounds__(kScanThreads)
void kda_fwd_scan_kernel(const Tin *__restrict__ v, const float *__restrict__ h0,
                         const int32_t *__restrict__ cu, const float *__restrict__ Tw,
                         const float *__restrict__ Ow, float *__restrict__ o, float *__restrict__ hT,
                         int64_t T, int H, int64_t chunks_per_seq, float scale)
{
    constexpr int LD = D + 4;          // rows 16-byte aligned: the operand tiles are written 16 bytes at a time
    extern __shared__ float smem[];
    float *sQ = smem, *sK = sQ + kC * LD, *sG = sK + kC * LD, *sA = sG + kC * LD;   // Gamma.Q, Gamma^{i->C}.K, Gamma.K, M | A_qk
    float *sV = sA + kC * kLA, *sVn = sV + kC * kBV;                 // V slice -> Y -> O, V_new
    float *sS = sVn + kC * kBV, *sGend = sS + D * kBV;               // state slice, G_C

    const int n = blockIdx.x, h = blockIdx.y, col0 = blockIdx.z * kBV, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t state_off = ((int64_t)n * H + h) * (int64_t)(D * D);
    for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
        const int d = idx / kBV, c = idx % kBV;
        sS[idx] = h0 ? h0[state_off + (int64_t)d * D + col0 + c] : 0.f;
    }

    const int64_t nchunks = (len + kC - 1) / kC;
    const int64_t slot_first = chunk_slot(cu, n, chunks_per_seq, 0) * H + h;
    auto valid_rows = [&](int64_t ci) { return (int)((len - ci * kC < kC) ? (len - ci * kC) : kC); };
    StepFetch<Tin, D, true> nxt;
    if (nchunks > 0)
        nxt.fetch(Ow + slot_first * (int64_t)operand_floats<D>(), v, Tw + (slot_first * 2 + 1) * (int64_t)kTile,
                  tok_base, valid_rows(0), H, h, col0, tid);
    for (int64_t ci = 0; ci < nchunks; ++ci) {
        const int nv = valid_rows(ci);
        const int64_t tok0 = tok_base + ci * kC;
        const int64_t slot = slot_first + ci * H;
        __syncthreads();
        nxt.commit(sQ, sK, sG, sA, sV, sGend, 1.f, tid);
        if (ci + 1 < nchunks)
            nxt.fetch(Ow + (slot + H) * (int64_t)operand_floats<D>(), v, Tw + ((slot + H) * 2 + 1) * (int64_t)kTile,
                      tok0 + kC, valid_rows(ci + 1), H, h, col0, tid);
        __syncthreads();
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        const int r0 = 16 * (wave & 3);
        const int cb = kTokCols == 2 ? 0 : 16 * (wave >> 2);
        f32x4 y[kTokCols] = {};
        mma16t<kTokCols>(0, D, g, y, [&](int k) { return sG[(r0 + m) * LD + k]; },                    // Kg S0
                         [&](int k, int c) { return sS[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)                       // Y = V - Kg S0
#pragma unroll
            for (int j = 0; j < 4; ++j) sV[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] -= y[c][j];
        __syncthreads();
        f32x4 vn[kTokCols] = {};
        mma16t<kTokCols>(0, r0 + 16, g, vn, [&](int k) { return k <= r0 + m ? sA[(r0 + m) * kLA + k] : 0.f; },   // Vn = M Y
                         [&](int k, int c) { return sV[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) sVn[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = vn[c][j];
        __syncthreads();
        f32x4 oo[kTokCols] = {};                                 // O = scale (Qg S0 + P Vn), P lower triangular
        mma16t<kTokCols>(0, D, g, oo, [&](int k) { return sQ[(r0 + m) * LD + k]; },
                         [&](int k, int c) { return sS[k * kBV + cb + 16 * c + m]; });
        mma16t<kTokCols>(0, r0 + 16, g, oo, [&](int k) { return k <= r0 + m ? sA[k * kLA + r0 + m + 1] : 0.f; },   // P[r0 + m][k]
                         [&](int k, int c) { return sVn[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)                       // staged in the dead Y tile
#pragma unroll
            for (int j = 0; j < 4; ++j) sV[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = scale * oo[c][j];
        __syncthreads();
        for (int idx = tid; idx < nv * kBV; idx += kScanThreads)
            o[((tok0 + idx / kBV) * H + h) * (int64_t)D + col0 + idx % kBV] = sV[idx];
        using ST = StateTiles<D>;
        for (int q = 0; q < ST::RPW; ++q) {                              // S1 = Diag(e^G_C) S0 + Kt^T Vn
            const int d0 = 16 * (ST::kPair ? wave * ST::RPW + q : wave % ST::NRT);
            const int sb = ST::kPair ? 0 : 16 * (wave / ST::NRT);
            f32x4 acc[ST::NC];
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[c][j] = sS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] * fast_exp2(sGend[d0 + 4 * g + j]);
            mma16t<ST::NC>(0, kC, g, acc, [&](int k) { return sK[k * LD + d0 + m]; },
                           [&](int k, int c) { return sVn[k * kBV + sb + 16 * c + m]; });
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j) sS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] = acc[c][j];
        }
    }
    if (hT) {
        __syncthreads();
        for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
            const int d = idx / kBV, c = idx % kBV;
            hT[state_off + (int64_t)d * D + col0 + c] = sS[idx];
        }
    }
}

// ------------------------------------------------------------------------------------------
// Backward walk with dS: dVn, dV = X, the dS1 of every chunk, dh0.
// ------------------------------------------------------------------------------------------
template <typename Tdo, int D>
__global__ __launch_bounds__(kScanThreads)
void kda_bwd_scan_kernel(const int32_t *__restrict__ cu, const float *__restrict__ Tw,
                         const float *__restrict__ Ow,
                         const Tdo *__restrict__ d_o, const float *__restrict__ d_hT,
                         float *__restrict__ dSc,
                         float *__restrict__ dVnw, float *__restrict__ dv, float *__restrict__ dh0,
                         int64_t T, int H, int64_t chunks_per_seq, float scale)
{
    constexpr int LD = D + 4;          // rows 16-byte aligned: the operand tiles are written 16 bytes at a time
    extern __shared__ float smem[];
    float *sQ = smem, *sK = sQ + kC * LD, *sG = sK + kC * LD, *sA = sG + kC * LD;
    float *sdO = sA + kC * kLA, *sdVn = sdO + kC * kBV, *sX = sdVn + kC * kBV;
    float *sdS = sX + kC * kBV, *sGend = sdS + D * kBV;

    const int n = blockIdx.x, h = blockIdx.y, col0 = blockIdx.z * kBV, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t state_off = ((int64_t)n * H + h) * (int64_t)(D * D);
    for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
        const int d = idx / kBV, c = idx % kBV;
        sdS[idx] = d_hT ? d_hT[state_off + (int64_t)d * D + col0 + c] : 0.f;
    }

    const int64_t nchunks = (len + kC - 1) / kC;
    const int64_t slot_first = chunk_slot(cu, n, chunks_per_seq, 0) * H + h;     // slots of a sequence are H apart
    auto valid_rows = [&](int64_t ci) { return (int)((len - ci * kC < kC) ? (len - ci * kC) : kC); };
    StepFetch<Tdo, D, true> nxt;
    if (nchunks > 0)
        nxt.fetch(Ow + (slot_first + (nchunks - 1) * H) * (int64_t)operand_floats<D>(), d_o,
                  Tw + ((slot_first + (nchunks - 1) * H) * 2 + 1) * (int64_t)kTile,
                  tok_base + (nchunks - 1) * kC, valid_rows(nchunks - 1), H, h, col0, tid);
    for (int64_t ci = nchunks - 1; ci >= 0; --ci) {
        const int nv = valid_rows(ci);
        const int64_t tok0 = tok_base + ci * kC;
        const int64_t slot = slot_first + ci * H;
        __syncthreads();
        for (int idx = tid; idx < D * kBV; idx += kScanThreads) {         // dS1 of this chunk
            const int d = idx / kBV, c = idx % kBV;
            dSc[slot * (int64_t)(D * D) + (int64_t)d * D + col0 + c] = sdS[idx];
        }
        nxt.commit(sQ, sK, sG, sA, sdO, sGend, scale, tid);
        if (ci > 0)                                              // the next chunk's loads fly during this one's work
            nxt.fetch(Ow + (slot - H) * (int64_t)operand_floats<D>(), d_o, Tw + ((slot - H) * 2 + 1) * (int64_t)kTile,
                      tok0 - kC, kC, H, h, col0, tid);
        __syncthreads();
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        const int r0 = 16 * (wave & 3);                          // this wave's 16 token rows ...
        const int cb = kTokCols == 2 ? 0 : 16 * (wave >> 2);     // ... and first slice column
        f32x4 dvn[kTokCols] = {};                                // dVn = Kt dS1 + P^T dO (P lower triangular)
        mma16t<kTokCols>(0, D, g, dvn, [&](int k) { return sK[(r0 + m) * LD + k]; },
                         [&](int k, int c) { return sdS[k * kBV + cb + 16 * c + m]; });
        mma16t<kTokCols>(r0, kC, g, dvn, [&](int k) { return k >= r0 + m ? sA[(r0 + m) * kLA + k + 1] : 0.f; },   // P[k][r0 + m]
                         [&](int k, int c) { return sdO[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) sdVn[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = dvn[c][j];
        __syncthreads();
        for (int idx = tid; idx < nv * kBV; idx += kScanThreads)         // whole 128-byte rows of the slice at a time
            dVnw[((tok0 + idx / kBV) * H + h) * (int64_t)D + col0 + idx % kBV] = sdVn[idx];
        f32x4 xx[kTokCols] = {};                                 // X = M^T dVn = dV
        mma16t<kTokCols>(r0, kC, g, xx, [&](int k) { return k >= r0 + m ? sA[k * kLA + r0 + m] : 0.f; },         // M[k][r0 + m]
                         [&](int k, int c) { return sdVn[k * kBV + cb + 16 * c + m]; });
#pragma unroll
        for (int c = 0; c < kTokCols; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) sX[(r0 + 4 * g + j) * kBV + cb + 16 * c + m] = xx[c][j];
        __syncthreads();
        for (int idx = tid; idx < nv * kBV; idx += kScanThreads)
            dv[((tok0 + idx / kBV) * H + h) * (int64_t)D + col0 + idx % kBV] = sX[idx];
        using ST = StateTiles<D>;
        for (int q = 0; q < ST::RPW; ++q) {                              // dS0
            const int d0 = 16 * (ST::kPair ? wave * ST::RPW + q : wave % ST::NRT);
            const int sb = ST::kPair ? 0 : 16 * (wave / ST::NRT);
            f32x4 acc[ST::NC];
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[c][j] = sdS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] * fast_exp2(sGend[d0 + 4 * g + j]);
            mma16t<ST::NC>(0, kC, g, acc, [&](int k) { return sQ[k * LD + d0 + m]; },
                           [&](int k, int c) { return sdO[k * kBV + sb + 16 * c + m]; });
            mma16t<ST::NC>(0, kC, g, acc, [&](int k) { return -sG[k * LD + d0 + m]; },
                           [&](int k, int c) { return sX[k * kBV + sb + 16 * c + m]; });
#pragma unroll
            for (int c = 0; c < ST::NC; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j) sdS[(d0 + 4 * g + j) * kBV + sb + 16 * c + m] = acc[c][j];
        }
    }
    if (dh0) {
        __syncthreads();
        for (int idx = tid; idx < D * kBV; idx += kScanThreads) {
            const int d = idx / kBV, c = idx % kBV;
            dh0[state_off + (int64_t)d * D + col0 + c] = sdS[idx];
        }
    }
}

// ------------------------------------------------------------------------------------------
// Per chunk: products with S0 and dS1, and the two C x C products.
// ------------------------------------------------------------------------------------------
constexpr int kProductsThreads = 512;

template <int D> constexpr size_t products_lds_floats()
{
    return (size_t)(D > 2 * kC ? D : 2 * kC) * (D + 1) + 2 * kC * (D + 1) + 2 * D + kProductsThreads;
}


// Row inside a 32 x 32 matrix-core accumulator tile of register j for a lane in half hh (the
// column is lane % 32).
__device__ __forceinline__ int acc_row32(int j, int hh) { return 8 * (j >> 2) + 4 * hh + (j & 3); }

// One 32 x 32 tile of  out[r][d] = sum_c sRow[r0 + r][c] * sCol[d0 + d][c]  on the matrix cores in
// fp32 (v_mfma_f32_32x32x2_f32: lane l feeds row l % 32 of both operands at contraction index
// k + l / 32).  Both operand tiles are [.][ld] floats in LDS.
template <int K>
__device__ __forceinline__ f32x16 tile_rows_times_rows(const float *sRow, const float *sCol, int ld, int lane)
{
    const float *pa = sRow + (lane & 31) * ld + (lane >> 5);
    const float *pb = sCol + (lane & 31) * ld + (lane >> 5);
    f32x16 acc = {};
#pragma unroll 8
    for (int k = 0; k < K; k += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], pb[k], acc, 0, 0, 0);
    return acc;
}

// out[r][d] = sum_c sOp[r][c] * sS[d][c] for all 64 rows and D columns: wave w of NT / 64 owns the
// tiles t = w, w + NT / 64, ... of the (64 / 32) x (D / 32) grid (numbered ti), column block
// t % (D / 32) -- so a lane sees one column d all along -- and hands every element to
// sink(ti, j, r, d, value), j the accumulator register.
template <int D, int NT, typename Sink>
__device__ __forceinline__ void times_state_t(const float *sOp, const float *sS, int tid, Sink &&sink)
{
    constexpr int LD = D + 1, NB = D / 32, NW = NT / 64, TPW = (2 * NB + NW - 1) / NW;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5;
#pragma unroll
    for (int ti = 0; ti < TPW; ++ti) {
        const int t = wave + NW * ti;
        if (t < 2 * NB) {
            const int d0 = 32 * (t % NB), r0 = 32 * (t / NB);
            const f32x16 acc = tile_rows_times_rows<D>(sOp + r0 * LD, sS + d0 * LD, LD, lane);
#pragma unroll
            for (int j = 0; j < 16; ++j) sink(ti, j, r0 + acc_row32(j, hh), d0 + (lane & 31), acc[j]);
        }
    }
}

// dst[r][i] = sum_c sR[r][c] * sI[i][c] for i <= r (row-major C x C in global memory): the three
// 32 x 32 tiles on or below the diagonal, one per wave.
template <int D>
__device__ __forceinline__ void lower_product(const float *sR, const float *sI, float *__restrict__ dst, int tid)
{
    constexpr int LD = D + 1;
    const int wave = tid >> 6, lane = tid & 63, hh = lane >> 5;
    if (wave < 3) {
        const int r0 = wave == 0 ? 0 : 32, i0 = wave == 2 ? 32 : 0;
        const f32x16 acc = tile_rows_times_rows<D>(sR + r0 * LD, sI + i0 * LD, LD, lane);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int r = r0 + acc_row32(j, hh), i = i0 + (lane & 31);
            if (i <= r) dst[r * kC + i] = acc[j];
        }
    }
}

template <typename Tin, typename Tdo, int D>
__global__ __launch_bounds__(kProductsThreads)
void kda_bwd_products_kernel(const Tin *__restrict__ q, const Tin *__restrict__ k,
                             const Tin *__restrict__ log_alpha, const int32_t *__restrict__ cu,
                             const Tdo *__restrict__ d_o, const float *__restrict__ Sc,
                             const float *__restrict__ dSc, const float *__restrict__ Yw,
                             const float *__restrict__ Vnw, const float *__restrict__ dVnw,
                             const float *__restrict__ dv, float *__restrict__ dq,
                             float *__restrict__ dk, float *__restrict__ dg, float *__restrict__ dgC,
                             float *__restrict__ Cw, int64_t T, int H, int64_t chunks_per_seq, float scale)
{
    constexpr int LD = D + 1, NT = kProductsThreads, RG = NT / D, NB = D / 32, NW = NT / 64;
    extern __shared__ float smem[];
    float *sS = smem;                       // [D][LD] S0, later dS1; later two [C][LD] operand tiles
    float *sOp = sS + (D > 2 * kC ? D : 2 * kC) * LD;   // [C][LD] row operand
    float *sG = sOp + kC * LD;              // [C][LD] G (log2 units)
    float *sGend = sG + kC * LD;            // [D]
    float *sgc = sGend + D;                 // [D]
    float *sPart = sgc + D;                 // [RG][D]

    const int64_t ci = blockIdx.y;
    const int n = blockIdx.x, h = blockIdx.z, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t c0 = ci * kC;
    if (c0 >= len) return;
    const int nv = (int)((len - c0 < kC) ? (len - c0) : kC);
    const int64_t tok0 = tok_base + c0;
    const int64_t slot = chunk_slot(cu, n, chunks_per_seq, ci) * H + h;
    const float *S0 = Sc + slot * (int64_t)(D * D);
    const float *dS1 = dSc + slot * (int64_t)(D * D);
    const int64_t base = (tok0 * H + h) * (int64_t)D, stride = (int64_t)H * D;
    auto load_rows = [&](float *dst, const float *src, float mul) {      // [C][D] token rows -> LDS
        rows_to_lds<float, kC, D, NT>(dst, LD, src + base, stride, nv, mul, tid);
    };
    auto load_state = [&](const float *src) {
        rows_to_lds<float, D / 2, D, NT>(sS, LD, src, D, D, 1.f, tid);
        rows_to_lds<float, D / 2, D, NT>(sS + (D / 2) * LD, LD, src + (D / 2) * D, D, D, 1.f, tid);
    };

    rows_to_lds<Tin, kC, D, NT>(sG, LD, log_alpha + base, stride, nv, kLog2e, tid);
    load_state(S0);
    rows_to_lds<Tdo, kC, D, NT>(sOp, LD, d_o + base, stride, nv, scale, tid);
    __syncthreads();
    cumsum_rows<D, NT>(sG, sPart, sGend, tid);

    // The three products below land on the same elements of every lane, so dq, dk and dG stay in
    // registers until all three are in and are written once.
    constexpr int TPW = (2 * NB + NW - 1) / NW;               // result tiles per wave
    f32x16 gq[TPW], gk[TPW], gg[TPW], kv[TPW];
    // dQg = dO S0^T:  dq = Gamma . dQg,  dG = dQg . Gamma . q
    times_state_t<D, NT>(sOp, sS, tid, [&](int ti, int j, int r, int d, float acc) {
        const int64_t off = ((tok0 + (r < nv ? r : 0)) * H + h) * (int64_t)D + d;
        const float t = acc * fast_exp2(sG[r * LD + d]);         // rows past nv: dO is zero there, so is t
        gq[ti][j] = t;
        gg[ti][j] = t * load_as_float(q + off);
        kv[ti][j] = load_as_float(k + off);
    });
    __syncthreads();
    load_rows(sOp, dv, 1.f);                                             // X
    __syncthreads();
    // dKg = -X S0^T:  dk = Gamma . dKg,  dG += dKg . Gamma . k
    times_state_t<D, NT>(sOp, sS, tid, [&](int ti, int j, int r, int d, float acc) {
        const float t = -acc * fast_exp2(sG[r * LD + d]);
        gk[ti][j] = t;
        gg[ti][j] = fmaf(t, kv[ti][j], gg[ti][j]);
    });
    __syncthreads();
    // dG_C (first part) = e^(G_C) . rowsum(dS1 . S0); dS1 is fetched once, multiplied into the S0 tile for
    // the row sums and kept in registers until it replaces that tile
    constexpr int kWords = D * D / 4 / NT;                               // 16-byte words of dS1 per thread
    uint4 ds[kWords];
#pragma unroll
    for (int u = 0; u < kWords; ++u) ds[u] = reinterpret_cast<const uint4 *>(dS1)[tid + NT * u];
#pragma unroll
    for (int u = 0; u < kWords; ++u) {
        const int idx = 4 * (tid + NT * u);
        float *p = sS + (idx / D) * LD + idx % D;
        p[0] *= __uint_as_float(ds[u].x); p[1] *= __uint_as_float(ds[u].y);
        p[2] *= __uint_as_float(ds[u].z); p[3] *= __uint_as_float(ds[u].w);
    }
    __syncthreads();
    if (tid < D) {
        float acc = 0.f;
        for (int c = 0; c < D; ++c) acc += sS[tid * LD + c];
        sgc[tid] = acc * fast_exp2(sGend[tid]);
    }
    load_rows(sOp, Vnw, 1.f);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kWords; ++u) {
        const int idx = 4 * (tid + NT * u);
        float *p = sS + (idx / D) * LD + idx % D;
        p[0] = __uint_as_float(ds[u].x); p[1] = __uint_as_float(ds[u].y);
        p[2] = __uint_as_float(ds[u].z); p[3] = __uint_as_float(ds[u].w);
    }
    __syncthreads();
    // dKt = Vn dS1^T:  dk += e^(G_C - G) . dKt,  dG -= dKt . Kt,  dG_C += sum_t dKt . Kt
    float gc_part = 0.f;
    times_state_t<D, NT>(sOp, sS, tid, [&](int ti, int j, int r, int d, float acc) {
        const float t = acc * fast_exp2(sGend[d] - sG[r * LD + d]);
        const float tk = t * kv[ti][j];                          // rows past nv: Vn and k are zero there
        gc_part += tk;
        if (r < nv) {
            const int64_t off = ((tok0 + r) * H + h) * (int64_t)D + d;
            dq[off] = gq[ti][j];
            dk[off] = gk[ti][j] + t;
            dg[off] = gg[ti][j] - tk;
        }
    });
    {   // a lane's elements all sit in column 32 (wave % NB) + lane % 32; NT / D lanes share a column
        const int wave = tid >> 6, lane = tid & 63;
        sPart[((lane >> 5) + 2 * (wave / NB)) * D + 32 * (wave % NB) + (lane & 31)] = gc_part;
    }
    __syncthreads();
    if (tid < D) {
        float acc = sgc[tid];
        for (int g = 0; g < RG; ++g) acc += sPart[g * D + tid];
        dgC[slot * D + tid] = acc;
    }
    // dP = Tril(dO Vn^T), dM = Tril(dVn Y^T): sOp holds Vn; the state area holds two row tiles
    float *sR = sS, *sI2 = sS + kC * LD;
    rows_to_lds<Tdo, kC, D, NT>(sR, LD, d_o + base, stride, nv, scale, tid);
    __syncthreads();
    lower_product<D>(sR, sOp, Cw + slot * (int64_t)(2 * kC * kC), tid);
    __syncthreads();
    load_rows(sR, dVnw, 1.f);
    load_rows(sI2, Yw, 1.f);
    __syncthreads();
    lower_product<D>(sR, sI2, Cw + slot * (int64_t)(2 * kC * kC) + kC * kC, tid);
}

// ------------------------------------------------------------------------------------------
// Per chunk: gradient through T, pairwise decay terms, dlog_alpha, dbeta.
// ------------------------------------------------------------------------------------------
constexpr int kChainThreads = 1024;

template <int D> constexpr size_t chain_lds_floats()
{
    return 3 * kC * (D + 1) + 3 * kC * kLA + 2 * kC + D + kChainThreads;
}

template <typename Tin, int D>
__global__ __launch_bounds__(kChainThreads)
void kda_bwd_chain_kernel(const Tin *__restrict__ q, const Tin *__restrict__ k,
                          const Tin *__restrict__ log_alpha, const Tin *__restrict__ beta,
                          const int32_t *__restrict__ cu, const float *__restrict__ Tw,
                          const float *__restrict__ Cw, const float *__restrict__ dgC,
                          float *__restrict__ dq,
                          float *__restrict__ dk, float *__restrict__ dla, float *__restrict__ dbeta,
                          int64_t T, int H, int64_t chunks_per_seq)
{
    constexpr int LD = D + 1, NT = kChainThreads, NW = NT / 64, RG = NT / D;
    constexpr int TG = 16 / RG < 4 ? 16 / RG : 4;           // tokens a thread takes together in the pairwise phase
    extern __shared__ float smem[];
    float *sQ = smem, *sK = sQ + kC * LD, *sG = sK + kC * LD;
    float *sA = sG + kC * LD;               // T - I (strict lower), A_kk (upper, transposed)
    float *sB = sA + kC * kLA;              // dM -> dT -> dL -> dA_kk (lower), dP (upper, transposed)
    float *sZ = sB + kC * kLA;              // dT T^T
    float *sBeta = sZ + kC * kLA, *sdb = sBeta + kC, *sGend = sdb + kC, *sTot = sGend + D;

    const int64_t ci = blockIdx.y;
    const int n = blockIdx.x, h = blockIdx.z, tid = threadIdx.x;
    int64_t tok_base, len;
    if (cu) { tok_base = cu[n]; len = (int64_t)cu[n + 1] - tok_base; }
    else    { tok_base = (int64_t)n * T; len = T; }
    const int64_t c0 = ci * kC;
    if (c0 >= len) return;
    const int nv = (int)((len - c0 < kC) ? (len - c0) : kC);
    const int64_t tok0 = tok_base + c0;
    const int64_t slot = chunk_slot(cu, n, chunks_per_seq, ci) * H + h;

    {   // dM (lower, diagonal included) and dP (stored transposed above the diagonal)
        const float *cP = Cw + slot * (int64_t)(2 * kC * kC), *cM = cP + kC * kC;
        BlockFetch<kC * kC / 4, NT> fp, fm;                         // all loads first (entries above the diagonal were
        fp.fetch(cP, tid);                                       // never written: read, not used)
        fm.fetch(cM, tid);
#pragma unroll
        for (int u = 0; u < kC * kC / 4 / NT; ++u) {
            const int idx = 4 * (tid + NT * u), r = idx >> 6, i0 = idx & 63;
            const float pv[4] = {__uint_as_float(fp.buf[u].x), __uint_as_float(fp.buf[u].y),
                                 __uint_as_float(fp.buf[u].z), __uint_as_float(fp.buf[u].w)};
            const float mv[4] = {__uint_as_float(fm.buf[u].x), __uint_as_float(fm.buf[u].y),
                                 __uint_as_float(fm.buf[u].z), __uint_as_float(fm.buf[u].w)};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i0 + e <= r) { sB[r * kLA + i0 + e] = mv[e]; sB[(i0 + e) * kLA + r + 1] = pv[e]; }
        }
    }
    load_tile<NT>(sA, Tw + slot * 2 * (int64_t)kTile, tid);
    chunk_load<Tin, D, NT>(q, k, log_alpha, beta, tok0, nv, H, h, sQ, sK, sG, sBeta, sGend, sTot, tid);

    auto Tm = [&](int r, int j) { return r == j ? 1.f : sA[r * kLA + j]; };   // r >= j

    // dbeta_j = sum_{r>=j} dM[r,j] T[r,j]
    if (tid < kC) {
        float acc = 0.f;
        for (int r = tid; r < kC; ++r) acc = fmaf(sB[r * kLA + tid], Tm(r, tid), acc);
        sdb[tid] = acc;
    }
    __syncthreads();
    // dT = dM Diag(beta)
    for (int idx = tid; idx < kC * kC; idx += NT) {
        const int r = idx >> 6, j = idx & 63;
        if (j <= r) sB[r * kLA + j] *= sBeta[j];
    }
    __syncthreads();
    // Z[a,i] = sum_{b <= min(a,i)} dT[a,b] T[i,b]: the 16 tiles of 16 x 16 spread over the waves
    {
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        for (int tile = wave; tile < 16; tile += NW) {
            const int Ab = tile & 3, Ib = tile >> 2;
            const int a = 16 * Ab + m, i = 16 * Ib + m;
            const f32x4 acc = mma16(0, 16 * ((Ab < Ib ? Ab : Ib) + 1), g, f32x4{0.f, 0.f, 0.f, 0.f},
                                    [&](int b_) { return b_ <= a ? sB[a * kLA + b_] : 0.f; },
                                    [&](int b_) { return b_ < i ? sA[i * kLA + b_] : (b_ == i ? 1.f : 0.f); });
#pragma unroll
            for (int j = 0; j < 4; ++j) sZ[(16 * Ab + 4 * g + j) * kLA + 16 * Ib + m] = acc[j];
        }
    }
    __syncthreads();
    // dL[r,i] = -sum_{a>=r} T[a,r] Z[a,i]  (i < r), then dbeta_r += sum_i dL A_kk, dA_kk = beta_r dL
    {
        const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
        for (int tile = wave; tile < 16; tile += NW) {
            const int Rb = tile & 3, Ib = tile >> 2;
            if (Ib > Rb) continue;
            const int r = 16 * Rb + m;
            const f32x4 acc = mma16(16 * Rb, kC, g, f32x4{0.f, 0.f, 0.f, 0.f},
                                    [&](int a_) { return a_ > r ? sA[a_ * kLA + r] : (a_ == r ? 1.f : 0.f); },
                                    [&](int a_) { return sZ[a_ * kLA + 16 * Ib + m]; });
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rr = 16 * Rb + 4 * g + j, ii = 16 * Ib + m;
                if (ii < rr) sB[rr * kLA + ii] = -acc[j];
            }
        }
    }
    __syncthreads();
    if (tid < kC) {
        const int r = tid;
        float acc = sdb[r];
        for (int i = 0; i < r; ++i) acc = fmaf(sB[r * kLA + i], sA[i * kLA + r + 1], acc);
        if (r < nv) dbeta[(tok0 + r) * H + h] = acc;
    }
    __syncthreads();
    for (int idx = tid; idx < kC * kC; idx += NT) {
        const int r = idx >> 6, i = idx & 63;
        if (i < r) sB[r * kLA + i] *= sBeta[r];
    }
    __syncthreads();

    // Decay terms, one 16-token block Bk at a time.  With a1[t] = sum_{i<t} dA_kk[t,i] k_i e^(G_t - G_i),
    // a2[t] the same with dP (i <= t), b1[t] = sum_{r>t} (dA_kk[r,t] k_r + dP[r,t] q_r) e^(G_r - G_t) (r >= t
    // for dP):  dq_t += a2,  dk_t += a1 + b1,  dG_t += k_t a1 + q_t a2 - k_t b1.  The parts of the sums
    // that cross a block boundary split the decay at the end E of the earlier block, e^(G_r - G_i) =
    // e^(G_r - E) e^(E - G_i) with both factors at most 1, and become block products on the matrix
    // cores (phase M, results staged in the dead T and Z tiles); the parts inside the block stay pair by
    // pair (phase P), which is also where everything is combined and written.
    const int d = tid % D, rg = tid / D;
    float dgt[kC / RG];
    float *stA1 = sA, *stA2 = sA + 16 * D, *stB1 = sZ;           // [16][D] each
#pragma unroll 1
    for (int Bk = 0; Bk < 4; ++Bk) {
        {   // ---- phase M: wave w takes the channel tiles dt = w, w + NT / 64, ...
            const int wave = tid >> 6, m = tid & 15, g = (tid >> 4) & 3;
            for (int dt = wave; dt < D / 16; dt += NW) {
                const int dc = 16 * dt + m;                      // this lane's channel as operand / result column
                f32x4 o1 = {0.f, 0.f, 0.f, 0.f}, o2 = {0.f, 0.f, 0.f, 0.f};
                for (int I = 0; I < Bk; ++I) {                   // tokens of block Bk as rows, earlier blocks as columns
                    const float E = sG[(16 * I + 15) * LD + dc];
                    f32x4 c1 = {0.f, 0.f, 0.f, 0.f}, c2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const int i = 16 * I + 4 * ks + g;
                        const float bv = sK[i * LD + dc] * fast_exp2(E - sG[i * LD + dc]);
                        c1 = __builtin_amdgcn_mfma_f32_16x16x4f32(sB[(16 * Bk + m) * kLA + i], bv, c1, 0, 0, 0);
                        c2 = __builtin_amdgcn_mfma_f32_16x16x4f32(sB[i * kLA + 16 * Bk + m + 1], bv, c2, 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float f = fast_exp2(sG[(16 * Bk + 4 * g + j) * LD + dc] - E);
                        o1[j] = fmaf(f, c1[j], o1[j]);
                        o2[j] = fmaf(f, c2[j], o2[j]);
                    }
                }
                const float E = sG[(16 * Bk + 15) * LD + dc];
                f32x4 cb = {0.f, 0.f, 0.f, 0.f};
                for (int R = Bk + 1; R < 4; ++R) {               // tokens of block Bk as columns, later blocks as rows
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const int r = 16 * R + 4 * ks + g;
                        const float f = fast_exp2(sG[r * LD + dc] - E);
                        cb = __builtin_amdgcn_mfma_f32_16x16x4f32(sB[r * kLA + 16 * Bk + m], sK[r * LD + dc] * f, cb, 0, 0, 0);
                        cb = __builtin_amdgcn_mfma_f32_16x16x4f32(sB[(16 * Bk + m) * kLA + r + 1], sQ[r * LD + dc] * f, cb, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int tl = 4 * g + j;
                    stA1[tl * D + dc] = o1[j];
                    stA2[tl * D + dc] = o2[j];
                    stB1[tl * D + dc] = cb[j] * fast_exp2(E - sG[(16 * Bk + tl) * LD + dc]);
                }
            }
        }
        __syncthreads();
        // ---- phase P: this thread's channel d and tokens 16 Bk + rg + RG jj, TG at a time
#pragma unroll 1
        for (int jj0 = 0; jj0 < 16 / RG; jj0 += TG) {
            int t_[TG];
            float Gt[TG], kt[TG], qt[TG], a1[TG], a2[TG], b1[TG];
#pragma unroll
            for (int u = 0; u < TG; ++u) {
                const int tl = rg + RG * (jj0 + u);
                t_[u] = 16 * Bk + tl;
                Gt[u] = sG[t_[u] * LD + d]; kt[u] = sK[t_[u] * LD + d]; qt[u] = sQ[t_[u] * LD + d];
                a1[u] = stA1[tl * D + d]; a2[u] = stA2[tl * D + d]; b1[u] = stB1[tl * D + d];
            }
            float old_q[TG], old_k[TG], old_g[TG];                  // what kda_bwd_products left: fetched now, used below
#pragma unroll
            for (int u = 0; u < TG; ++u) {
                const int64_t off = ((tok0 + (t_[u] < nv ? t_[u] : 0)) * H + h) * (int64_t)D + d;
                old_q[u] = dq[off]; old_k[u] = dk[off]; old_g[u] = dla[off];
            }
            for (int i = 16 * Bk; i < t_[TG - 1]; ++i) {              // the tokens as rows: columns i < t inside the block
                const float gi = sG[i * LD + d], ki = sK[i * LD + d];
#pragma unroll
                for (int u = 0; u < TG; ++u) {
                    const float kk = i < t_[u] ? ki * fast_exp2(Gt[u] - gi) : 0.f;
                    a1[u] = fmaf(sB[t_[u] * kLA + i], kk, a1[u]);
                    a2[u] = fmaf(sB[i * kLA + t_[u] + 1], kk, a2[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < TG; ++u) {
                a2[u] = fmaf(sB[t_[u] * kLA + t_[u] + 1], kt[u], a2[u]);     // dP[t,t]
                b1[u] = fmaf(sB[t_[u] * kLA + t_[u] + 1], qt[u], b1[u]);
            }
            for (int r = t_[0] + 1; r < 16 * Bk + 16; ++r) {     // the tokens as columns: rows r > t inside the block
                const float gr = sG[r * LD + d], kr = sK[r * LD + d], qr = sQ[r * LD + d];
#pragma unroll
                for (int u = 0; u < TG; ++u) {
                    const float e = r > t_[u] ? fast_exp2(gr - Gt[u]) : 0.f;
                    b1[u] = fmaf(fmaf(sB[r * kLA + t_[u]], kr, sB[t_[u] * kLA + r + 1] * qr), e, b1[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < TG; ++u) {
                float gsum = 0.f;
                if (t_[u] < nv) {
                    const int64_t off = ((tok0 + t_[u]) * H + h) * (int64_t)D + d;
                    dq[off] = old_q[u] + a2[u];
                    dk[off] = old_k[u] + a1[u] + b1[u];
                    gsum = old_g[u] + kt[u] * a1[u] + qt[u] * a2[u] - kt[u] * b1[u];
                }
                dgt[(16 * Bk) / RG + jj0 + u] = gsum;
            }
        }
        __syncthreads();
    }
    __syncthreads();
#pragma unroll 1
    for (int j = 0; j < kC / RG; ++j) sQ[(rg + RG * j) * LD + d] = dgt[j];
    __syncthreads();
    // dlog_alpha_t = sum_{r>=t} dG_r + dG_C
    if (tid < D) {
        float run = dgC[slot * D + tid];
        for (int r = nv - 1; r >= 0; --r) {
            run += sQ[r * LD + tid];
            dla[((tok0 + r) * H + h) * (int64_t)D + tid] = run;
        }
    }
}

template <typename F>
static kda_status reserve(F kern, size_t lds, const char *name)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess)
        return fail(KDA_ERR_LAUNCH, "%s: cannot reserve %zu B of LDS: %s", name, lds, hipGetErrorString(e));
    return KDA_OK;
}

struct BwdPlan {
    int64_t chunks_per_seq, max_chunks, nslots, ntok;
    size_t off_S, off_dS, off_Y, off_Vn, off_dVn, off_gC, off_C, off_T, off_O, total;
};

static BwdPlan bwd_plan(const kda_dims *d, bool packed)
{
    BwdPlan p{};
    const int64_t D = d->dk;
    p.chunks_per_seq = (d->seqlen + kC - 1) / kC;
    const int64_t longest = packed ? ((d->max_seqlen > 0 && d->max_seqlen < d->seqlen) ? d->max_seqlen : d->seqlen)
                                   : d->seqlen;
    p.max_chunks = (longest + kC - 1) / kC;
    const int64_t slots = packed ? d->seqlen / kC + d->num_seqs : (int64_t)d->num_seqs * p.chunks_per_seq;
    p.nslots = slots * d->heads;
    p.ntok = (packed ? d->seqlen : (int64_t)d->batch * d->seqlen) * d->heads;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    size_t at = 0;
    p.off_S = at;   at = up(at + (size_t)p.nslots * D * D * 4);
    p.off_dS = at;  at = up(at + (size_t)p.nslots * D * D * 4);
    p.off_Y = at;   at = up(at + (size_t)p.ntok * D * 4);
    p.off_Vn = at;  at = up(at + (size_t)p.ntok * D * 4);
    p.off_dVn = at; at = up(at + (size_t)p.ntok * D * 4);
    p.off_gC = at;  at = up(at + (size_t)p.nslots * D * 4);
    p.off_C = at;   at = up(at + (size_t)p.nslots * 2 * kC * kC * 4);
    p.off_T = at;   at = up(at + (size_t)p.nslots * 2 * kTile * 4);
    p.off_O = at;   at = up(at + (size_t)p.nslots * (3 * kC * D + D) * 4);
    p.total = at;
    return p;
}

template <typename Tin, typename Tdo, int D>
static kda_status launch_bwd(const kda_dims *dm, const BwdPlan &p, const void *q_, const void *k_,
                             const void *v_, const void *la_, const void *beta_, const float *h0,
                             const int32_t *cu, const void *d_o_, const float *d_hT, float *dq,
                             float *dk, float *dv, float *dla, float *dbeta, float *dh0, char *ws,
                             hipStream_t stream)
{
    const Tin *q = static_cast<const Tin *>(q_), *k = static_cast<const Tin *>(k_);
    const Tin *v = static_cast<const Tin *>(v_), *la = static_cast<const Tin *>(la_);
    const Tin *beta = static_cast<const Tin *>(beta_);
    const Tdo *d_o = static_cast<const Tdo *>(d_o_);
    float *Sc = reinterpret_cast<float *>(ws + p.off_S), *dSc = reinterpret_cast<float *>(ws + p.off_dS);
    float *Yw = reinterpret_cast<float *>(ws + p.off_Y), *Vnw = reinterpret_cast<float *>(ws + p.off_Vn);
    float *dVnw = reinterpret_cast<float *>(ws + p.off_dVn), *gC = reinterpret_cast<float *>(ws + p.off_gC);
    float *Cw = reinterpret_cast<float *>(ws + p.off_C), *Tw = reinterpret_cast<float *>(ws + p.off_T);
    float *Ow = reinterpret_cast<float *>(ws + p.off_O);

    const size_t lds_scan = scan_lds_floats<D>() * 4, lds_states = states_lds_floats<D>() * 4,
                 lds_prod = products_lds_floats<D>() * 4,
                 lds_chain = chain_lds_floats<D>() * 4, lds_prep = prep_lds_floats<D>() * 4;
    kda_status st;
    if ((st = reserve(kda_bwd_prep_kernel<Tin, D>, lds_prep, "kda_bwd_prep")) != KDA_OK) return st;
    if ((st = reserve(kda_bwd_states_kernel<Tin, D>, lds_states, "kda_bwd_states")) != KDA_OK) return st;
    if ((st = reserve(kda_bwd_scan_kernel<Tdo, D>, lds_scan, "kda_bwd_scan")) != KDA_OK) return st;
    if ((st = reserve(kda_bwd_products_kernel<Tin, Tdo, D>, lds_prod, "kda_bwd_products")) != KDA_OK) return st;
    if ((st = reserve(kda_bwd_chain_kernel<Tin, D>, lds_chain, "kda_bwd_chain")) != KDA_OK) return st;

    const int H = dm->heads;
    const int64_t T = dm->seqlen;
    const dim3 gscan((unsigned)dm->num_seqs, (unsigned)H, (unsigned)(D / kBV));
    const dim3 gchunk((unsigned)dm->num_seqs, (unsigned)p.max_chunks, (unsigned)H);
    if (p.max_chunks > 0)
        hipLaunchKernelGGL((kda_bwd_prep_kernel<Tin, D>), gchunk, dim3(kPrepThreads), lds_prep, stream, q, k, la, beta, cu,
                           Tw, Ow, T, H, p.chunks_per_seq);
    hipLaunchKernelGGL((kda_bwd_states_kernel<Tin, D>), gscan, dim3(kScanThreads), lds_states, stream, v, h0, cu, Tw, Ow,
                       Sc, Yw, Vnw, T, H, p.chunks_per_seq);
    hipLaunchKernelGGL((kda_bwd_scan_kernel<Tdo, D>), gscan, dim3(kScanThreads), lds_scan, stream, cu, Tw, Ow,
                       d_o, d_hT, dSc, dVnw, dv, dh0, T, H, p.chunks_per_seq, dm->scale);
    if (p.max_chunks > 0) {
        hipLaunchKernelGGL((kda_bwd_products_kernel<Tin, Tdo, D>), gchunk, dim3(kProductsThreads), lds_prod, stream, q, k, la, cu,
                           d_o, Sc, dSc, Yw, Vnw, dVnw, dv, dq, dk, dla, gC, Cw, T, H, p.chunks_per_seq,
                           dm->scale);
        hipLaunchKernelGGL((kda_bwd_chain_kernel<Tin, D>), gchunk, dim3(kChainThreads), lds_chain, stream, q, k, la, beta,
                           cu, Tw, Cw, gC, dq, dk, dla, dbeta, T, H, p.chunks_per_seq);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_chunk_bwd: %s", hipGetErrorString(e));
    return KDA_OK;
}

struct FwdPlan { int64_t chunks_per_seq, max_chunks, nslots; size_t off_T, off_O, total; };

static FwdPlan fwd_plan(const kda_dims *d, bool packed)
{
    const BwdPlan b = bwd_plan(d, packed);
    FwdPlan p{};
    p.chunks_per_seq = b.chunks_per_seq; p.max_chunks = b.max_chunks; p.nslots = b.nslots;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    p.off_T = 0;
    p.off_O = up((size_t)p.nslots * 2 * kTile * 4);
    p.total = up(p.off_O + (size_t)p.nslots * (3 * kC * d->dk + d->dk) * 4);
    return p;
}

template <typename Tin, int D>
static kda_status launch_fwd(const kda_dims *dm, const FwdPlan &p, const void *q_, const void *k_, const void *v_,
                             const void *la_, const void *beta_, const float *h0, const int32_t *cu, float *o,
                             float *hT, char *ws, hipStream_t stream)
{
    float *Tw = reinterpret_cast<float *>(ws + p.off_T), *Ow = reinterpret_cast<float *>(ws + p.off_O);
    const size_t lds_prep = prep_lds_floats<D>() * 4, lds_scan = fwd_scan_lds_floats<D>() * 4;
    kda_status st;
    if ((st = reserve(kda_bwd_prep_kernel<Tin, D>, lds_prep, "kda_bwd_prep")) != KDA_OK) return st;
    if ((st = reserve(kda_fwd_scan_kernel<Tin, D>, lds_scan, "kda_fwd_scan")) != KDA_OK) return st;
    const int H = dm->heads;
    if (p.max_chunks > 0)
        hipLaunchKernelGGL((kda_bwd_prep_kernel<Tin, D>), dim3((unsigned)dm->num_seqs, (unsigned)p.max_chunks, (unsigned)H),
                           dim3(kPrepThreads), lds_prep, stream, static_cast<const Tin *>(q_),
                           static_cast<const Tin *>(k_), static_cast<const Tin *>(la_),
                           static_cast<const Tin *>(beta_), cu, Tw, Ow, (int64_t)dm->seqlen, H, p.chunks_per_seq);
    hipLaunchKernelGGL((kda_fwd_scan_kernel<Tin, D>), dim3((unsigned)dm->num_seqs, (unsigned)H, (unsigned)(D / kBV)),
                       dim3(kScanThreads), lds_scan, stream, static_cast<const Tin *>(v_), h0, cu, Tw, Ow, o, hT,
                       (int64_t)dm->seqlen, H, p.chunks_per_seq, dm->scale);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "fp32 prefill: %s", hipGetErrorString(e));
    return KDA_OK;
}

}  // namespace

// The size entry points do not see cu_seqlens.  A batch of one row may or may not come with it, and the
// packed layout (one extra slot per sequence) is the larger of the two, so a single row is sized as packed:
// whatever the dispatcher then lays out fits.
static bool sized_as_packed(const kda_dims *d) { return d->num_seqs != d->batch || d->batch == 1; }

size_t chunk_bwd_workspace_size(const kda_dims *d)
{
    return bwd_plan(d, sized_as_packed(d)).total;
}

kda_status chunk_bwd_dispatch(const kda_dims *dm, const void *q, const void *k, const void *v,
                              const void *log_alpha, const void *beta, const float *h0,
                              const int32_t *cu, const void *d_o, const float *d_hT, float *dq,
                              float *dk, float *dv, float *dla, float *dbeta, float *dh0,
                              void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const BwdPlan p = bwd_plan(dm, cu != nullptr);
    // (the size the library reports is the requirement, even where this call's own layout is smaller)
    const size_t need = chunk_bwd_workspace_size(dm) > p.total ? chunk_bwd_workspace_size(dm) : p.total;
    if (need > workspace_bytes || (need && !workspace))
        return fail(KDA_ERR_WORKSPACE, "kda_chunk_bwd needs %zu B of workspace, got %zu", need, workspace_bytes);
    if (p.max_chunks > 65535)
        return fail(KDA_ERR_UNSUPPORTED, "kda_chunk_bwd: sequences longer than %d tokens", 65535 * kC);
    char *ws = static_cast<char *>(workspace);
    const bool bf = dm->in_dtype == KDA_BF16;
#define KDA_BWD(TIN, TDO, DD) launch_bwd<TIN, TDO, DD>(dm, p, q, k, v, log_alpha, beta, h0, cu, d_o, d_hT, dq, dk, dv, \
                                                       dla, dbeta, dh0, ws, stream)
    // d_o has dims->out_dtype: fp32, or bf16 (bf16 inputs only)
    if (dm->out_dtype == KDA_BF16)
        return dm->dk == 128 ? KDA_BWD(__hip_bfloat16, __hip_bfloat16, 128) : KDA_BWD(__hip_bfloat16, __hip_bfloat16, 64);
    if (dm->dk == 128) return bf ? KDA_BWD(__hip_bfloat16, float, 128) : KDA_BWD(float, float, 128);
    return bf ? KDA_BWD(__hip_bfloat16, float, 64) : KDA_BWD(float, float, 64);
#undef KDA_BWD
}

// The fp32 prefill from kda_bwd_prep and kda_fwd_scan.  Workspace: the two packed tiles and the three
// operand tiles per (chunk, head).  0 if the shape is outside what the grid can hold (then the
// single-kernel path of kda_chunk_f32.hip serves).
size_t chunk_f32_fast_workspace_size(const kda_dims *d)
{
    const FwdPlan p = fwd_plan(d, sized_as_packed(d));
    return p.max_chunks > 65535 ? 0 : p.total;
}

kda_status chunk_f32_fast_dispatch(const kda_dims *dm, const void *q, const void *k, const void *v,
                                   const void *log_alpha, const void *beta, const float *h0,
                                   const int32_t *cu, void *o, float *hT, void *workspace, hipStream_t stream)
{
    const FwdPlan p = fwd_plan(dm, cu != nullptr);
    char *ws = static_cast<char *>(workspace);
    float *of = static_cast<float *>(o);
    const bool bf = dm->in_dtype == KDA_BF16;
#define KDA_FWD(TIN, DD) launch_fwd<TIN, DD>(dm, p, q, k, v, log_alpha, beta, h0, cu, of, hT, ws, stream)
    if (dm->dk == 128) return bf ? KDA_FWD(__hip_bfloat16, 128) : KDA_FWD(float, 128);
    return bf ? KDA_FWD(__hip_bfloat16, 64) : KDA_FWD(float, 64);
#undef KDA_FWD
}

}  // namespace kda
