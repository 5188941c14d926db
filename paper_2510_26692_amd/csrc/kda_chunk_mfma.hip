// Chunkwise KDA prefill on the matrix cores (Section 3.1) for bf16 inputs,
// d_k = d_v = 128, C = 64.
//
// Two kernels per time segment:
//
//  kda_intra  one workgroup per (chunk, head), all chunks in parallel.  It forms the
//             running log-decay G, the two intra-chunk matrices A_kk and A_qk, the
//             UT-transform M = (I + StrictTril(Diag(beta) A_kk))^-1 Diag(beta) by
//             forward substitution, W = M (Gamma.K), U = M V and the decay-scaled
//             operands Gamma.Q and Gamma^{i->C}.K, and leaves them in the workspace
//             in MFMA register order (kda_mfma_layout.h).
//  kda_scan   one workgroup per (sequence, head), sequential over that sequence's
//             chunks: V_new = U - W S, O = (Gamma.Q) S + Tril(A_qk) V_new,
//             S <- Diag(gamma^C) S + (Gamma^{i->C}.K)^T V_new, with the fp32 state
//             held in accumulator registers for the whole sequence.
//
// With up to a third of the compute units' worth of (sequence, head) pairs the two kernels run
// at the same time (kda_intra on a helper stream, each slot handed over through a flag); with
// very few pairs and long sequences kda_scan_split takes the place of kda_scan and cuts the
// chunk axis into ranges that several workgroups walk side by side (the chunk recurrence is
// affine in the state).  Optional fused stages (Section 4): the input prologue in kda_intra, the
// output gate in kda_scan.
//
// Matrix-core operands are fp16 (unit roundoff 2^-11), accumulation is fp32.  The
// raw bf16 inputs convert to fp16 exactly; only derived operands are rounded.
//
// Decay handling ("secondary chunking"): the chunk is cut into four 16-token
// sub-chunks.  For a pair of tokens in different sub-chunks the decay
// 2^(G_r - G_i) is split at the boundary in front of the row's sub-chunk, so both
// factors are <= 1 and go straight into the operands.  Inside a sub-chunk it is
// split at the point where half of the sub-chunk's decay D (in log2 units) has been
// spent: row factor 2^(G_r + D/2), column factor 2^(-G_i - D/2), both within
// 2^(+-D/2), so fp16 holds them for D up to kStrongLog2 (the row operands of all
// tiles carry the 2^(D/2) and the column operands of the tiles below undo it).  A
// channel whose decay across the sub-chunk exceeds 2^-kStrongLog2 keeps the split at
// the sub-chunk's start, is taken out of the diagonal tile's column operand and is
// added back exactly, pair by pair, in fp32.
#include <stdlib.h>
#include <type_traits>

#include <mutex>

#include "kda_common.h"
#include "kda_mfma_layout.h"

namespace kda {

extern int g_phase_mask;   // diagnostics switches owned by kda_api.hip
extern int g_overlap;
extern int g_split;
extern double g_split_ratio;

namespace mfma {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kStrongLog2 = 24.0f;   // sub-chunk decay below 2^-24 leaves the fast operands
constexpr float kRowScale = 4.0f;      // keeps small row operands out of the fp16 subnormals
constexpr float kRowShift = 2.0f;      // log2(kRowScale)

// ----------------------------------------------------------------------------------
// LDS map of kda_intra (bytes).  Regions are reused as the phases advance; the whole
// map stays under 80 KiB so that two workgroups share a compute unit.
// ----------------------------------------------------------------------------------
constexpr int kLdH = 136;                               // halfs per row of a [64][128] fp16 tile
constexpr int kTileH = 64 * kLdH * 2;                   // 17408 B
constexpr int kLdF = 68;                                // floats per row of a [64][64] fp32 tile
constexpr int kTileF = 64 * kLdF * 4;                   // 17408 B
constexpr int kLdM = 72;                                // halfs per row of a [64][64] fp16 tile
constexpr int kTileM = 64 * kLdM * 2;                   // 9216 B

constexpr int kX = 0;                                   // fp32 (I + L)^-1
constexpr int kTab = kX;                                //   early alias: per-channel constants, 7 x [4][128] fp32
constexpr int kFix = kTab + 7 * 2048;                   //   early alias: scratch of the strong-channel fix-up
constexpr int kL = kX + kTileF;                         // fp32 L = StrictTril(Diag(beta) A_kk), stored transposed
constexpr int kAq = kL + kTileF;                        // fp16 Tril(A_qk), stored transposed
constexpr int kColS = kL;                               //   early alias: column operands [6 tiles][4][64] x 16 B
constexpr int kV = kL;                                  //   late alias: fp16 V tile
constexpr int kGK = kAq + kTileM;                       // fp16 Gamma.K
constexpr int kKp = kGK + kTileH;                       // fp16 Gamma^{i->C}.K
constexpr int kM = kKp;                                 //   late alias: fp16 M
constexpr int kTot = kKp + kTileH;                      // fp32 [4][128] sub-chunk log2-decay totals
constexpr int kBeta = kTot + 4 * 128 * 4;               // fp32 [64]
constexpr int kStrong = kBeta + 64 * 4;                 // u32 [4][4] strong-channel masks per (sub-chunk, g)
constexpr int kIntraLds = kStrong + 64;
static_assert(kFix + 4 * 4 * 16 * 3 * 4 <= kL, "early aliases must fit under X");
static_assert(kColS + 6 * 4 * 64 * 16 <= kGK, "early aliases must fit under L and A_qk");
static_assert(kIntraLds <= 80 * 1024, "kda_intra must leave room for two workgroups per CU");

// Half of a sub-chunk's log2 decay `tot` (<= 0), as a non-negative shift; 0 for a strong channel.
__device__ __forceinline__ float half_shift(float tot) { return (tot < -kStrongLog2) ? 0.f : -0.5f * tot; }

__device__ __forceinline__ uint32_t pack_h2(float a, float b)
{
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// lane i of each row of 16 lanes receives the value of lane i - N (0 when there is none)
template <int N> __device__ __forceinline__ float row_shr(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x110 + N, 0xf, 0xf, true));
}

// Transposing LDS read (ds_read_b64_tr_b16): `block` points at element (row 0, column 0) of a
// 4 x 16 block of 16-bit values with `ld` values between rows, the same for the 16 lanes of a group
// (lanes 16 i .. 16 i + 15).  Lane c of the group receives column c of rows 0..3, i.e. the four
// values an MFMA operand wants in consecutive contraction slots.  (Lane p hands the hardware the
// address of row p / 4, columns 4 (p % 4) .. + 3; it returns to lane c element c % 4 of the four
// rows handed in by lanes c / 4, 4 + c / 4, 8 + c / 4, 12 + c / 4.)
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x2 lds_read_tr4(const uint8_t *block, int ld, int lane)
{
    const int p = lane & 15;
    const uint8_t *a = block + ((p >> 2) * ld + 4 * (p & 3)) * 2;
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)a);
    return __builtin_bit_cast(u32x2, v);
}

// Workspace slots are written and read through buffer instructions with the device-scope cache
// policy (sc1): the stores write through the L2 of the writing XCD and the loads do not trust
// the L2 of the reading XCD, so a slot produced by one workgroup can be consumed by another one
// of a kernel that runs at the same time, with no cache write-back or invalidate in between.
// The descriptor covers exactly one slot; offsets beyond it are dropped by the hardware.
constexpr int kCacheDevice = 16;                            // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slot_resource(const uint8_t *slot)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(slot), 0, kSlotBytes, 0x00020000);
}
template <int kPolicy, typename V> __device__ __forceinline__ void slot_store16(__amdgpu_buffer_rsrc_t rs, int off, V val)
{
    static_assert(sizeof(V) == 16, "16-byte store");
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, val), rs, off, 0, kPolicy);
}
template <int kPolicy, typename V> __device__ __forceinline__ void slot_store8(__amdgpu_buffer_rsrc_t rs, int off, V val)
{
    static_assert(sizeof(V) == 8, "8-byte store");
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, val), rs, off, 0, kPolicy);
}
template <int kPolicy> __device__ __forceinline__ u32x4 slot_load16(__amdgpu_buffer_rsrc_t rs, int off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kPolicy);
}

// ----------------------------------------------------------------------------------
// kda_intra
// ----------------------------------------------------------------------------------
// Lane (m = lane % 16, g = lane / 16) of wave R owns token 16 R + m and the 32 channels
// 32 ks + 8 g + e (ks = 0..3, e = 0..7): exactly its A/B operand slots of the 16x16x32 MFMA,
// so the decay-scaled operands of the A-matrix products are built in registers.
// kHandoff: the slot is handed to a kda_scan that runs at the same time (write-through stores and a
// ready flag); otherwise the stores are ordinary ones and the kernel boundary publishes them.
// kScalar: log_alpha is [B,T,H], one decay per (token, head) shared by all channels (the scalar-gate
// special case of Eq. (1), Section 2.2); the decay then leaves the matrix-core operands altogether.
// kRaw: q, k, log_alpha and beta arrive as the raw projections of Section 4 ("Neural
// Parameterization") and the kernel applies L2Norm to q and k, Sigmoid to beta and the decay
// function log alpha = -a_scale[h] softplus(gate + dt_bias[h][c]) itself, in fp32.
struct RawParams {
    const float *a_scale;    // [H] or NULL (= 1)
    const float *dt_bias;    // [H][128] or NULL (= 0)
    float eps;               // L2Norm: x / sqrt(sum x^2 + eps)
};

// log2(alpha) of one channel from its gate logit x (bias already added): -a * log2(1 + e^x)
__device__ __forceinline__ float log2_alpha_from_gate(float x, float a)
{
    const float t = x * kLog2e;
    const float sp = (t > 30.f) ? t : __log2f(1.f + fast_exp2(t));
    return -a * sp;
}

template <bool kHandoff, bool kRaw, bool kScalar = false>
__global__ __launch_bounds__(256, 2)
void kda_intra_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
                      const uint16_t *__restrict__ v, const uint16_t *__restrict__ log_alpha,
                      const uint16_t *__restrict__ beta, const int32_t *__restrict__ cu_seqlens,
                      uint8_t *__restrict__ ws, int64_t T, int H, int64_t seg_chunks,
                      int64_t seg_index, float scale, uint32_t *ready, uint32_t epoch, RawParams raw,
                      int parts, int part_len, int part0_len, const uint16_t *__restrict__ out_gate,
                      uint8_t *__restrict__ gate_ws)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // (the wave index is the same in all lanes: telling the compiler so turns the per-wave cases
    // below into scalar branches instead of masked vector code)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    constexpr int kPolicy = kHandoff ? kCacheDevice : 0;

    // Workgroup -> (head, sequence, chunk) straight from the 3-D grid (no divisions).  x = head;
    // with kHandoff y = sequence and z = chunk, so that workgroups are dispatched by chunk index
    // first and the slots a concurrently running kda_scan needs next are produced first;
    // otherwise y = chunk and z = sequence (consecutive workgroups write consecutive slots).
    const int h = (int)blockIdx.x;
    const int n = (int)(kHandoff ? blockIdx.y : blockIdx.z);
    // (when the scan is time-split into `parts` ranges -- the first of `part0_len` chunks, the others
    // of `part_len` -- its first phase walks all ranges but the last side by side, so the chunk
    // order interleaves those and lets the last range follow)
    int64_t cl = kHandoff ? blockIdx.z : blockIdx.y;
    if (kHandoff && parts > 1) {
        const unsigned first = (unsigned)(parts - 1), z = blockIdx.z;
        if (z < first * (unsigned)part_len) {
            const unsigned r = z % first, j = z / first;
            if (r == 0 && j >= (unsigned)part0_len) return;  // the first range is the shorter one
            cl = (r == 0) ? (int64_t)j : (int64_t)part0_len + (int64_t)(r - 1) * part_len + j;
        } else {
            cl = (int64_t)part0_len + (int64_t)(first - 1) * part_len + (z - first * (unsigned)part_len);
        }
    }
    if (cl >= seg_chunks) return;
    const int64_t slot = n * seg_chunks + cl;
    const int64_t ci = seg_index * seg_chunks + cl;
    int64_t tok_base, len;
    if (cu_seqlens) { tok_base = cu_seqlens[n]; len = (int64_t)cu_seqlens[n + 1] - tok_base; }
    else            { tok_base = (int64_t)n * T; len = T; }
    if (ci * kChunk >= len) return;                      // uniform for the workgroup
    const int nv = (int)((len - ci * kChunk < kChunk) ? (len - ci * kChunk) : kChunk);
    const int64_t tok0 = tok_base + ci * kChunk;
    const __amdgpu_buffer_rsrc_t out = slot_resource(ws + (slot * H + h) * (int64_t)kSlotBytes);

    float *sTot = reinterpret_cast<float *>(lds + kTot);
    float *sBeta = reinterpret_cast<float *>(lds + kBeta);
    uint32_t *sStrong = reinterpret_cast<uint32_t *>(lds + kStrong);
    float *sTab = reinterpret_cast<float *>(lds + kTab);     // [7][4][128]: P, E, Tinv, iA, iB, shifted total, row shift

    const int R = wave, m = lane & 15, g = lane >> 4;
    const int tok = 16 * R + m;

    // ---- output gate (fused epilogue): the chunk's gate logits are re-laid into the accumulator
    // order of the sequential kernel, which reads them like any other part of the slot.  The loads
    // go out first and the stores follow the kernel's own loads, so the copy hides in their latency.
    u32x4 ograw[4];
    if (out_gate) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
            u32x4 x = {0, 0, 0, 0};
            if (tokv < nv)
                x = *reinterpret_cast<const u32x4 *>(out_gate + ((tok0 + tokv) * H + h) * (int64_t)D + 8 * cg);
            ograw[i] = x;
        }
    }

    // ---- loads: 16 bytes (8 channels) per ks and tensor ----
    // (log_alpha first: the running sum below waits for it, k and q are not needed before B2)
    u32x4 kraw[4], qraw[4], graw[4];
    {
        const u32x4 z = {0, 0, 0, 0};
        const int64_t off = ((tok0 + tok) * H + h) * (int64_t)D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            graw[ks] = (!kScalar && tok < nv) ? *reinterpret_cast<const u32x4 *>(log_alpha + off + 32 * ks) : z;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kraw[ks] = (tok < nv) ? *reinterpret_cast<const u32x4 *>(k + off + 32 * ks) : z;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qraw[ks] = (tok < nv) ? *reinterpret_cast<const u32x4 *>(q + off + 32 * ks) : z;
    }
    static_assert(!(kRaw && kScalar), "the fused prologue is built for the per-channel gate");
    float gscalar = 0.f;                                     // kScalar: log alpha of this lane's token
    if (kScalar && tok < nv) gscalar = bf16_bits_to_float(log_alpha[(tok0 + tok) * H + h]);
    if (tid < kChunk) {
        float b = (tid < nv) ? bf16_bits_to_float(beta[(tok0 + tid) * H + h]) : 0.f;
        if (kRaw) b = (tid < nv) ? __builtin_amdgcn_rcpf(1.f + fast_exp2(-b * kLog2e)) : 0.f;   // Sigmoid
        sBeta[tid] = b;
    }
    if (out_gate) {
        // piece (token, 8 columns 8 cg ..) = column group q = cg % 4 of tile (token / 32, cg / 4): its
        // first four columns belong to lane (token % 32, hh = 0), the other four to lane (.., hh = 1)
        const __amdgpu_buffer_rsrc_t gout = __builtin_amdgcn_make_buffer_rsrc(
            gate_ws + (slot * H + h) * (int64_t)kGateSlotBytes, 0, kGateSlotBytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
            const int base = ((tokv >> 5) * 4 + (cg >> 2)) * kGateTileBytes + ((cg & 3) >> 1) * 1024 + (tokv & 31) * 16 +
                             (cg & 1) * 8;
            const u32x2 lo = {ograw[i][0], ograw[i][1]}, hi = {ograw[i][2], ograw[i][3]};
            slot_store8<kPolicy>(gout, base, lo);
            slot_store8<kPolicy>(gout, base + 32 * 16, hi);
        }
    }
    // kRaw: 1 / |q|, 1 / |k| of this lane's token (the four lanes g = 0..3 of a token hold 32 channels each)
    float invq = 1.f, invk = 1.f;
    if (kRaw) {
        float sq = 0.f, sk = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float a, b;
                unpack_bf16x2(kraw[ks][w], a, b); sk = fmaf(a, a, fmaf(b, b, sk));
                unpack_bf16x2(qraw[ks][w], a, b); sq = fmaf(a, a, fmaf(b, b, sq));
            }
        sq += __shfl_xor(sq, 16); sk += __shfl_xor(sk, 16);
        sq += __shfl_xor(sq, 32); sk += __shfl_xor(sk, 32);
        invq = (tok < nv) ? __builtin_amdgcn_rsqf(sq + raw.eps) : 0.f;
        invk = (tok < nv) ? __builtin_amdgcn_rsqf(sk + raw.eps) : 0.f;
    }

    f32x4 res_kk[4], res_qk[4];              // A_kk, A_qk tiles (R, I), I = 0..R
    if constexpr (kScalar) {
        // ---- scalar gate: A[r][i] = (k_r . k_i) 2^(G_r - G_i), so the tiles are plain K K^T and Q K^T
        // products of the fp16 copies of k and q (exact: they come from bf16), and the decay, at most
        // 1 where it is kept, multiplies the fp32 results.  Gamma.K, Gamma.Q and Gamma^{i->C}.K are k and q
        // times one factor per token.  No sub-chunk split and no exact path are needed.
        float *sG = reinterpret_cast<float *>(lds + kTab);   // [64] running log2 decay over the chunk
        float gs = gscalar * kLog2e;
        gs += row_shr<1>(gs); gs += row_shr<2>(gs); gs += row_shr<4>(gs); gs += row_shr<8>(gs);
        if (lane == 15) sTot[R] = gs;                        // total of sub-chunk R
        __syncthreads();                                                           // B1
        const float t0 = sTot[0], t1 = sTot[1], t2 = sTot[2], t3 = sTot[3];
        const float total = t0 + t1 + t2 + t3;
        const float Gc = gs + ((R > 0) ? t0 : 0.f) + ((R > 1) ? t1 : 0.f) + ((R > 2) ? t2 : 0.f);
        if (g == 0) sG[tok] = Gc;
        const float gam = fast_exp2(Gc), gam_end = fast_exp2(total - Gc), gam_q = gam * scale;
        if (R == 0) {   // gamma^C, the same for every channel
            const float gce = fast_exp2(total);
            slot_store8<kPolicy>(out, kOffGc + 2 * lane * 4, make_float2(gce, gce));
        }
        h8 rowK[4], rowQ[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            float kf[8], qf[8];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                unpack_bf16x2(kraw[ks][w], kf[2 * w], kf[2 * w + 1]);
                unpack_bf16x2(qraw[ks][w], qf[2 * w], qf[2 * w + 1]);
            }
            u32x4 t;
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(kf[2 * w], kf[2 * w + 1]);
            rowK[ks] = __builtin_bit_cast(h8, t);
            // the same k is the column operand of every tile below this sub-chunk
            if (R < 3) *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 1) * R / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
            if (R < 2) *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 2) * (R + 1) / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
            if (R < 1) *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 3) * (R + 2) / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(qf[2 * w], qf[2 * w + 1]);
            rowQ[ks] = __builtin_bit_cast(h8, t);
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(kf[2 * w] * gam, kf[2 * w + 1] * gam);
            *reinterpret_cast<u32x4 *>(lds + kGK + (tok * kLdH + 32 * ks + 8 * g) * 2) = t;
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(kf[2 * w] * gam_end, kf[2 * w + 1] * gam_end);
            *reinterpret_cast<u32x4 *>(lds + kKp + (tok * kLdH + 32 * ks + 8 * g) * 2) = t;
            {   // Gamma.Q to the workspace in MFMA register order (see the per-channel path)
                const uint32_t a0 = pack_h2(qf[0] * gam_q, qf[1] * gam_q), a1 = pack_h2(qf[2] * gam_q, qf[3] * gam_q);
                const uint32_t b0 = pack_h2(qf[4] * gam_q, qf[5] * gam_q), b1 = pack_h2(qf[6] * gam_q, qf[7] * gam_q);
                const bool odd = g & 1;
                const uint32_t r0 = __shfl_xor(odd ? a0 : b0, 16), r1 = __shfl_xor(odd ? a1 : b1, 16);
                u32x4 o4;
                if (odd) { o4[0] = r0; o4[1] = r1; o4[2] = b0; o4[3] = b1; }
                else     { o4[0] = a0; o4[1] = a1; o4[2] = r0; o4[3] = r1; }
                slot_store16<kPolicy>(out, kOffQp + frag_rts(tok >> 5, ks, g >> 1) * kFragBytes + ((tok & 31) + 32 * (g & 1)) * 16, o4);
            }
        }
        {
            f32x4 akk = {0.f, 0.f, 0.f, 0.f}, aqk = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                akk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowK[ks], rowK[ks], akk, 0, 0, 0);
                aqk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowQ[ks], rowK[ks], aqk, 0, 0, 0);
            }
            res_kk[R] = akk; res_qk[R] = aqk;
        }
        __syncthreads();                                                           // B3 (colS, sG visible)
#pragma unroll
        for (int I = 0; I < 3; ++I) {
            if (I < R) {
                f32x4 akk = {0.f, 0.f, 0.f, 0.f}, aqk = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const h8 b = *reinterpret_cast<const h8 *>(lds + kColS + (((R * (R - 1) / 2 + I) * 4 + ks) * 64 + lane) * 16);
                    akk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowK[ks], b, akk, 0, 0, 0);
                    aqk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowQ[ks], b, aqk, 0, 0, 0);
                }
                res_kk[I] = akk; res_qk[I] = aqk;
            }
        }
        // the decay 2^(G_r - G_i) on every kept entry (r >= i; the others are masked below)
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            if (I <= R) {
                const float gi = sG[16 * I + m];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float dlt = sG[16 * R + 4 * g + j] - gi;
                    const float f = fast_exp2(dlt < 0.f ? dlt : 0.f);
                    res_kk[I][j] *= f; res_qk[I][j] *= f;
                }
            }
        }
        __syncthreads();                                                           // B4 (early aliases dead)
    } else {
    // ---- G: running sum of log2(alpha) over the 16 tokens of the sub-chunk (lanes of a row) ----
    float G[32];
    f32x4 bias[8];                                           // kRaw: dt_bias of this lane's 32 channels
    float a_scale = 1.f;
    if (kRaw) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 8; ++i)
            bias[i] = raw.dt_bias ? *reinterpret_cast<const f32x4 *>(raw.dt_bias + h * D + 32 * (i >> 1) + 8 * g + 4 * (i & 1)) : z;
        if (raw.a_scale) a_scale = raw.a_scale[h];
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float a, b;
            unpack_bf16x2(graw[ks][w], a, b);
            if (kRaw) {
                // padding tokens must stay identity transitions: log alpha = 0
                const float b0 = bias[2 * ks + (w >> 1)][2 * (w & 1)], b1 = bias[2 * ks + (w >> 1)][2 * (w & 1) + 1];
                a = (tok < nv) ? log2_alpha_from_gate(a + b0, a_scale) : 0.f;
                b = (tok < nv) ? log2_alpha_from_gate(b + b1, a_scale) : 0.f;
            } else {
                a *= kLog2e; b *= kLog2e;
            }
            a += row_shr<1>(a); b += row_shr<1>(b);
            a += row_shr<2>(a); b += row_shr<2>(b);
            a += row_shr<4>(a); b += row_shr<4>(b);
            a += row_shr<8>(a); b += row_shr<8>(b);
            G[ks * 8 + 2 * w] = a; G[ks * 8 + 2 * w + 1] = b;
        }
    if (m == 15) {          // the last token of the sub-chunk holds its totals
        uint32_t smask = 0;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            f32x4 t0 = {G[ks * 8 + 0], G[ks * 8 + 1], G[ks * 8 + 2], G[ks * 8 + 3]};
            f32x4 t1 = {G[ks * 8 + 4], G[ks * 8 + 5], G[ks * 8 + 6], G[ks * 8 + 7]};
            *reinterpret_cast<f32x4 *>(sTot + R * 128 + 32 * ks + 8 * g) = t0;
            *reinterpret_cast<f32x4 *>(sTot + R * 128 + 32 * ks + 8 * g + 4) = t1;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (G[ks * 8 + e] < -kStrongLog2) smask |= 1u << (ks * 8 + e);
        }
        sStrong[R * 4 + g] = smask;
    }
    __syncthreads();                                                               // B1

    // ---- per-channel constants of sub-chunk R, two channels per lane ----
    {
        const int c2 = 2 * lane;
        float t0[4], t1[4];
#pragma unroll
        for (int J = 0; J < 4; ++J) {
            const float2 x = *reinterpret_cast<const float2 *>(sTot + J * 128 + c2);
            t0[J] = x.x; t1[J] = x.y;
        }
        float pre0 = 0.f, pre1 = 0.f, post0 = 0.f, post1 = 0.f;
#pragma unroll
        for (int J = 0; J < 4; ++J) {
            if (J < R) { pre0 += t0[J]; pre1 += t1[J]; }
            if (J > R) { post0 += t0[J]; post1 += t1[J]; }
        }
        // r1..r3 = R+1..R+3 (only used when they exist).  sh: the half-decay shift carried by the row
        // operands of sub-chunk R; the column operands of a tile (Rp, R) undo the shift of Rp.  The
        // column base value already undoes the shift of R+1 (n1), so the other constants put it back.
        const int r1 = (R + 1) & 3, r2 = (R + 2) & 3, r3 = (R + 3) & 3;
        const float sh0 = half_shift(t0[R]), sh1 = half_shift(t1[R]);
        const float n10 = (R < 3) ? half_shift(t0[r1]) : 0.f, n11 = (R < 3) ? half_shift(t1[r1]) : 0.f;
        float *tb = sTab + R * 128 + c2;
        // (the row operands carry kRowScale as +kRowShift in their exponent: tables 0, 5 and 6 account
        // for it; a strong channel is kept out of the diagonal tile's column operand by Tinv = 0)
        *reinterpret_cast<float2 *>(tb + 0 * 512) = make_float2(fast_exp2(pre0 - sh0 - kRowShift), fast_exp2(pre1 - sh1 - kRowShift));
        *reinterpret_cast<float2 *>(tb + 1 * 512) = make_float2(fast_exp2(post0 + n10), fast_exp2(post1 + n11));
        *reinterpret_cast<float2 *>(tb + 2 * 512) = make_float2((t0[R] < -kStrongLog2) ? 0.f : fast_exp2(-t0[R] - sh0 + n10),
                                                                (t1[R] < -kStrongLog2) ? 0.f : fast_exp2(-t1[R] - sh1 + n11));
        *reinterpret_cast<float2 *>(tb + 3 * 512) = make_float2(fast_exp2(t0[r1] - half_shift(t0[r2]) + n10),
                                                                fast_exp2(t1[r1] - half_shift(t1[r2]) + n11));
        *reinterpret_cast<float2 *>(tb + 4 * 512) = make_float2(fast_exp2(t0[r1] + t0[r2] - half_shift(t0[r3]) + n10),
                                                                fast_exp2(t1[r1] + t1[r2] - half_shift(t1[r3]) + n11));
        *reinterpret_cast<float2 *>(tb + 5 * 512) = make_float2(t0[R] + sh0 - n10 + kRowShift, t1[R] + sh1 - n11 + kRowShift);
        *reinterpret_cast<float2 *>(tb + 6 * 512) = make_float2(sh0 + kRowShift, sh1 + kRowShift);
        if (R == 0) {   // gamma^C: decay of the whole chunk
            float2 gc = make_float2(fast_exp2(t0[0] + t0[1] + t0[2] + t0[3]), fast_exp2(t1[0] + t1[1] + t1[2] + t1[3]));
            slot_store8<kPolicy>(out, kOffGc + c2 * 4, gc);
        }
    }
    uint32_t strong_all = 0;        // union over g of this sub-chunk's strong-channel slots
    {
        const uint32_t s0 = sStrong[R * 4 + 0], s1 = sStrong[R * 4 + 1], s2 = sStrong[R * 4 + 2],
                       s3 = sStrong[R * 4 + 3];
        strong_all = s0 | s1 | s2 | s3;
    }
    __syncthreads();                                                               // B2

    // the row shift goes into G once (a strong channel's shift is the constant kRowShift alone, so
    // the fix-up below, which uses differences of G, still sees its plain running sums)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const f32x4 x = *reinterpret_cast<const f32x4 *>(sTab + 6 * 512 + R * 128 + 32 * (i >> 1) + 8 * g + 4 * (i & 1));
#pragma unroll
        for (int z = 0; z < 4; ++z) G[4 * i + z] += x[z];
    }

    // ---- operands, built in registers ----
    h8 rowK[4], rowQ[4], colKd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        float kf[8], qf[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            unpack_bf16x2(kraw[ks][w], kf[2 * w], kf[2 * w + 1]);
            unpack_bf16x2(qraw[ks][w], qf[2 * w], qf[2 * w + 1]);
        }
        if (kRaw) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { kf[e] *= invk; qf[e] *= invq; }
        }
        const int cb = R * 128 + 32 * ks + 8 * g;
        float tot[8], P[8], E[8], Ti[8], iA[8], iB[8];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(sTab + 5 * 512 + cb + 4 * hf);
            const f32x4 b = *reinterpret_cast<const f32x4 *>(sTab + 0 * 512 + cb + 4 * hf);
            const f32x4 c = *reinterpret_cast<const f32x4 *>(sTab + 1 * 512 + cb + 4 * hf);
            const f32x4 d = *reinterpret_cast<const f32x4 *>(sTab + 2 * 512 + cb + 4 * hf);
#pragma unroll
            for (int z = 0; z < 4; ++z) { tot[4 * hf + z] = a[z]; P[4 * hf + z] = b[z]; E[4 * hf + z] = c[z]; Ti[4 * hf + z] = d[z]; }

            if (R <= 1) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(sTab + 3 * 512 + cb + 4 * hf);
#pragma unroll
                for (int z = 0; z < 4; ++z) iA[4 * hf + z] = x[z];
            }
            if (R == 0) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(sTab + 4 * 512 + cb + 4 * hf);
#pragma unroll
                for (int z = 0; z < 4; ++z) iB[4 * hf + z] = x[z];
            }
        }
        float rk[8], rq[8], cs[8], cd[8], gk[8], qp[8], kp[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float Ge = G[ks * 8 + e];
            const float rf = fast_exp2(Ge);                       // kRowScale 2^(G_r + D/2): within kRowScale 2^(+-D/2)
            const float sf = fast_exp2(tot[e] - Ge);              // decay from this token to the end of R, less the shift of R+1
            rk[e] = kf[e] * rf;
            rq[e] = qf[e] * rf;
            cs[e] = kf[e] * sf;
            cd[e] = cs[e] * Ti[e];                                // k 2^(-G_i - D/2); 0 for a strong channel
            gk[e] = rk[e] * P[e];                                 // Gamma . K
            qp[e] = rq[e] * (P[e] * scale);                       // scale * Gamma . Q
            kp[e] = cs[e] * E[e];                                 // Gamma^{i->C} . K
        }
        u32x4 t;
#pragma unroll
        for (int w = 0; w < 4; ++w) t[w] = pack_h2(rk[2 * w], rk[2 * w + 1]);
        rowK[ks] = __builtin_bit_cast(h8, t);
#pragma unroll
        for (int w = 0; w < 4; ++w) t[w] = pack_h2(rq[2 * w], rq[2 * w + 1]);
        rowQ[ks] = __builtin_bit_cast(h8, t);
#pragma unroll
        for (int w = 0; w < 4; ++w) t[w] = pack_h2(cd[2 * w], cd[2 * w + 1]);
        colKd[ks] = __builtin_bit_cast(h8, t);
        // column operands for the sub-chunks below: tile (Rp, R) splits the decay at the boundary in
        // front of sub-chunk Rp, so the part across the sub-chunks in between rides on the columns
        if (R < 3) {
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(cs[2 * w], cs[2 * w + 1]);
            *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 1) * R / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
        }
        if (R < 2) {
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(cs[2 * w] * iA[2 * w], cs[2 * w + 1] * iA[2 * w + 1]);
            *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 2) * (R + 1) / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
        }
        if (R < 1) {
#pragma unroll
            for (int w = 0; w < 4; ++w) t[w] = pack_h2(cs[2 * w] * iB[2 * w], cs[2 * w + 1] * iB[2 * w + 1]);
            *reinterpret_cast<u32x4 *>(lds + kColS + ((((R + 3) * (R + 2) / 2 + R) * 4 + ks) * 64 + lane) * 16) = t;
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) t[w] = pack_h2(gk[2 * w], gk[2 * w + 1]);
        *reinterpret_cast<u32x4 *>(lds + kGK + (tok * kLdH + 32 * ks + 8 * g) * 2) = t;
#pragma unroll
        for (int w = 0; w < 4; ++w) t[w] = pack_h2(kp[2 * w], kp[2 * w + 1]);
        *reinterpret_cast<u32x4 *>(lds + kKp + (tok * kLdH + 32 * ks + 8 * g) * 2) = t;
        // Gamma.Q goes straight to the workspace in MFMA register order: lanes g and g^1 swap one
        // 4-channel piece each so that every lane ends up with a complete 16-byte slot
        {
            const uint32_t a0 = pack_h2(qp[0], qp[1]), a1 = pack_h2(qp[2], qp[3]);
            const uint32_t b0 = pack_h2(qp[4], qp[5]), b1 = pack_h2(qp[6], qp[7]);
            const bool odd = g & 1;
            const uint32_t r0 = __shfl_xor(odd ? a0 : b0, 16), r1 = __shfl_xor(odd ? a1 : b1, 16);
            u32x4 o4;
            if (odd) { o4[0] = r0; o4[1] = r1; o4[2] = b0; o4[3] = b1; }
            else     { o4[0] = a0; o4[1] = a1; o4[2] = r0; o4[3] = r1; }
            slot_store16<kPolicy>(out, kOffQp + frag_rts(tok >> 5, ks, g >> 1) * kFragBytes + ((tok & 31) + 32 * (g & 1)) * 16, o4);
        }
    }

    // ---- A_kk, A_qk tiles of sub-chunk row R on the matrix cores (16x16, K = 128) ----
    {
        f32x4 akk = {0.f, 0.f, 0.f, 0.f}, aqk = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            akk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowK[ks], colKd[ks], akk, 0, 0, 0);
            aqk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowQ[ks], colKd[ks], aqk, 0, 0, 0);
        }
        akk *= (1.0f / kRowScale);
        aqk *= (1.0f / kRowScale);
        if (strong_all) {
            // channels left out of colKd: exact pairwise terms 2^(G_r - G_i) in fp32.  For each
            // register slot with a strong channel the 64 lanes drop (G, k, q) of that slot into a
            // small scratch indexed [g][token]; every lane then reads column m and its four rows.
            float *fix = reinterpret_cast<float *>(lds + kFix) + wave * (4 * 16 * 3);
            // (a run-time loop over the register slots that hold a strong channel: the slot's values
            // are picked by compare-and-select, so the rare path stays a few hundred instructions)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                uint32_t bits = __builtin_amdgcn_readfirstlane((strong_all >> (ks * 8)) & 0xffu);
                while (bits) {
                    const int e = __builtin_ctz(bits);
                    bits &= bits - 1;
                    float Ge = G[ks * 8];
#pragma unroll
                    for (int z = 1; z < 8; ++z) Ge = (e == z) ? G[ks * 8 + z] : Ge;
                    uint32_t kw = kraw[ks][0], qw = qraw[ks][0];
#pragma unroll
                    for (int z = 1; z < 4; ++z) {
                        kw = ((e >> 1) == z) ? kraw[ks][z] : kw;
                        qw = ((e >> 1) == z) ? qraw[ks][z] : qw;
                    }
                    const float kfe = invk * ((e & 1) ? __uint_as_float(kw & 0xffff0000u) : __uint_as_float(kw << 16));
                    const float qfe = invq * ((e & 1) ? __uint_as_float(qw & 0xffff0000u) : __uint_as_float(qw << 16));
                    const int sl = ks * 8 + e;
                    __builtin_amdgcn_wave_barrier();
                    fix[(g * 16 + m) * 3 + 0] = Ge;
                    fix[(g * 16 + m) * 3 + 1] = kfe;
                    fix[(g * 16 + m) * 3 + 2] = qfe;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                        if ((sStrong[R * 4 + gg] >> sl) & 1u) {
                            const float Gi = fix[(gg * 16 + m) * 3 + 0], ki = fix[(gg * 16 + m) * 3 + 1];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int rr = 4 * g + j;
                                if (rr >= m) {
                                    const float t = ki * fast_exp2(fix[(gg * 16 + rr) * 3 + 0] - Gi);
                                    akk[j] = fmaf(fix[(gg * 16 + rr) * 3 + 1], t, akk[j]);
                                    aqk[j] = fmaf(fix[(gg * 16 + rr) * 3 + 2], t, aqk[j]);
                                }
                            }
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
        }
        res_kk[R] = akk; res_qk[R] = aqk;
    }
    __syncthreads();                                                               // B3 (colS visible)
#pragma unroll
    for (int I = 0; I < 3; ++I) {
        if (I < R) {
            f32x4 akk = {0.f, 0.f, 0.f, 0.f}, aqk = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const h8 b = *reinterpret_cast<const h8 *>(lds + kColS + (((R * (R - 1) / 2 + I) * 4 + ks) * 64 + lane) * 16);
                akk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowK[ks], b, akk, 0, 0, 0);
                aqk = __builtin_amdgcn_mfma_f32_16x16x32_f16(rowQ[ks], b, aqk, 0, 0, 0);
            }
            res_kk[I] = akk * (1.0f / kRowScale);
            res_qk[I] = aqk * (1.0f / kRowScale);
        }
    }
    __syncthreads();                                                               // B4 (early aliases dead)

    }

    // ---- L and Tril(A_qk) tiles of row R; fp16 V tile ----
    {
        // (L is kept transposed, sLT[column][row]: a lane's four rows of a column are contiguous, one
        // 16-byte store per tile, and the substitution below reads a column of L as a row)
        float *sLT = reinterpret_cast<float *>(lds + kL);
        // (Tril(A_qk) likewise, sAqT[column][row] in fp16: 8-byte stores here, transposing reads below)
        uint16_t *sAqT = reinterpret_cast<uint16_t *>(lds + kAq);
        const f32x4 beta4 = *reinterpret_cast<const f32x4 *>(sBeta + 16 * R + 4 * g);
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            const int i = 16 * I + m;                       // column token of this lane
            u32x2 av = {0u, 0u};
            if (I <= R) {
                f32x4 lv;
                float qv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 16 * R + 4 * g + j;
                    lv[j] = (i < r) ? beta4[j] * res_kk[I][j] : 0.f;
                    qv[j] = (i <= r) ? res_qk[I][j] * scale : 0.f;
                }
                *reinterpret_cast<f32x4 *>(sLT + i * kLdF + 16 * R + 4 * g) = lv;
                av[0] = pack_h2(qv[0], qv[1]); av[1] = pack_h2(qv[2], qv[3]);
            }
            *reinterpret_cast<u32x2 *>(sAqT + i * kLdM + 16 * R + 4 * g) = av;   // zeros above the diagonal tiles
        }
    }
    __syncthreads();                                                               // B5

    // V is fetched now; its latency hides behind the UT transform
    u32x4 vraw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
        u32x4 x = {0, 0, 0, 0};
        if (tokv < nv)
            x = *reinterpret_cast<const u32x4 *>(v + ((tok0 + tokv) * H + h) * (int64_t)D + 8 * cg);
        vraw[i] = x;
    }

    // ---- UT transform, diagonal 16x16 blocks: column j of (I + L_ww)^-1 per lane ----
    {
        // (column by column: once x[i] is final, the updates of the rows below it are independent
        // of one another, so the dependent chain is 16 long instead of 120; each x[r] still
        // receives its terms in the order i = 0, 1, ..)
        const float *sLT = reinterpret_cast<const float *>(lds + kL);
        float *sX = reinterpret_cast<float *>(lds + kX);
        const int j = lane & 15, w = wave;
        float x[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = (r == j) ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < 15; ++i) {
            const float *col = sLT + (16 * w + i) * kLdF + 16 * w;      // L[16 w + r][16 w + i], r = 0..15
            const float xi = x[i];
#pragma unroll
            for (int r = i + 1; r < 16; ++r) x[r] = fmaf(-col[r], xi, x[r]);
        }
        if (lane < 16) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sX[(16 * w + r) * kLdF + 16 * w + j] = x[r];
        }
    }
    // ---- copy (Gamma^{i->C}.K)^T out in MFMA register order ----
    {
        // lane (x = lane % 32, hh): channel 32 tau + x, tokens 32 rho + kidx(s, hh, 0..7), which are two
        // runs of four consecutive tokens: two transposing reads per fragment
        const int hh = lane >> 5, xb = 16 * ((lane >> 4) & 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = wave * 4 + i;                     // Kt frag f = (tau*2 + rho)*2 + s
            const int tau = f >> 2, rho = (f >> 1) & 1, s = f & 1;
            const uint8_t *blk = lds + kKp + ((32 * rho + kidx(s, hh, 0)) * kLdH + 32 * tau + xb) * 2;
            const u32x2 lo = lds_read_tr4(blk, kLdH, lane), hi = lds_read_tr4(blk + 8 * kLdH * 2, kLdH, lane);
            u32x4 o4 = {lo[0], lo[1], hi[0], hi[1]};
            slot_store16<kPolicy>(out, kOffKt + f * kFragBytes + lane * 16, o4);
        }
    }
    __syncthreads();                                                               // B6

    // ---- UT transform, off-diagonal blocks: X_RI = -X_RR sum_{I<=J<R} L_RJ X_JI (fp32 MFMA) ----
    {
        const float *sLT = reinterpret_cast<const float *>(lds + kL);
        float *sX = reinterpret_cast<float *>(lds + kX);
        for (int Rr = 1; Rr < 4; ++Rr) {
            if (wave < Rr) {
                const int Ii = wave;
                f32x4 t = {0.f, 0.f, 0.f, 0.f};
                for (int J = Ii; J < Rr; ++J) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const float a = sLT[(16 * J + 4 * ks + g) * kLdF + 16 * Rr + m];   // L[16 Rr + m][16 J + 4 ks + g]
                        const float b = sX[(16 * J + 4 * ks + g) * kLdF + 16 * Ii + m];
                        t = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, t, 0, 0, 0);
                    }
                }
                // second product with contraction slot (ks, g) standing for index 4 g + ks, so
                // that register ks of the accumulator t is the B operand as it stands
                f32x4 r = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const float a = sX[(16 * Rr + m) * kLdF + 16 * Rr + 4 * g + ks];
                    r = __builtin_amdgcn_mfma_f32_16x16x4f32(a, t[ks], r, 0, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) sX[(16 * Rr + 4 * g + j) * kLdF + 16 * Ii + m] = -r[j];
            }
            __syncthreads();                                                       // B7
        }
    }

    // ---- M = X Diag(beta) as fp16 (over the dead K' tile); Tril(A_qk) out; V tile (over L) ----
    {
        const float *sX = reinterpret_cast<const float *>(lds + kX);
        _Float16 *sM = reinterpret_cast<_Float16 *>(lds + kM);
        // four consecutive columns per thread and pass: 16-byte reads, 8-byte writes
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int idx = tid + 256 * pass, r = idx >> 4, j0 = 4 * (idx & 15);
            const f32x4 xr = *reinterpret_cast<const f32x4 *>(sX + r * kLdF + j0);
            const f32x4 br = *reinterpret_cast<const f32x4 *>(sBeta + j0);
            float val[4];
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const int j = j0 + z;
                val[z] = (j < r) ? xr[z] * br[z] : ((j == r) ? br[z] : 0.f);
            }
            u32x2 w2 = {pack_h2(val[0], val[1]), pack_h2(val[2], val[3])};
            *reinterpret_cast<u32x2 *>(sM + r * kLdM + j0) = w2;
        }
        // lane (x, hh) of fragment (rr, ri, s): row token 32 rr + x, column tokens 32 ri + 16 s + 4 hh + 0..3
        // and + 8..11, which are rows of the transposed tile
        const int hh = lane >> 5, xb = 16 * ((lane >> 4) & 1);
        for (int idx = wave; idx < 6; idx += 4) {
            const int p = idx >> 1, s = idx & 1;
            const int rr = (p == 0) ? 0 : 1, ri = (p == 2) ? 1 : 0;
            const uint8_t *blk = lds + kAq + ((32 * ri + 16 * s + 4 * hh) * kLdM + 32 * rr + xb) * 2;
            const u32x2 a = lds_read_tr4(blk, kLdM, lane), b = lds_read_tr4(blk + 8 * kLdM * 2, kLdM, lane);
            u32x4 o4 = {a[0], a[1], b[0], b[1]};
            slot_store16<kPolicy>(out, kOffAqk + frag_aqk(rr, ri, s) * kFragBytes + lane * 16, o4);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
            u32x4 y;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float a, b;
                unpack_bf16x2(vraw[i][w], a, b);
                y[w] = pack_h2(a, b);
            }
            *reinterpret_cast<u32x4 *>(lds + kV + (tokv * kLdH + 8 * cg) * 2) = y;
        }
    }
    __syncthreads();                                                               // B8

    // ---- W^T = (Gamma.K)^T M^T (wave = d_k tile) and U = M V (wave = d_v tile) ----
    {
        // operands with the tokens in the contraction slots: lane (x, hh) wants channel 32 wave + x of
        // the eight tokens 16 s4 + 8 hh + 0..7 of the [token][channel] tiles: two transposing reads each
        const int x = lane & 31, hh = lane >> 5, xb = 16 * ((lane >> 4) & 1);
        h8 mf[2][4], gk[4], vv[4];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
            for (int rho = 0; rho < 2; ++rho)
                mf[rho][s4] = *reinterpret_cast<const h8 *>(lds + kM + ((32 * rho + x) * kLdM + 16 * s4 + 8 * hh) * 2);
            const int off = ((16 * s4 + 8 * hh) * kLdH + 32 * wave + xb) * 2;
            const u32x2 g0 = lds_read_tr4(lds + kGK + off, kLdH, lane), g1 = lds_read_tr4(lds + kGK + off + 4 * kLdH * 2, kLdH, lane);
            const u32x2 v0 = lds_read_tr4(lds + kV + off, kLdH, lane), v1 = lds_read_tr4(lds + kV + off + 4 * kLdH * 2, kLdH, lane);
            u32x4 pg = {g0[0], g0[1], g1[0], g1[1]}, pv = {v0[0], v0[1], v1[0], v1[1]};
            gk[s4] = __builtin_bit_cast(h8, pg);
            vv[s4] = __builtin_bit_cast(h8, pv);
        }
#pragma unroll
        for (int rho = 0; rho < 2; ++rho) {
            f32x16 wt = {0.f}, u = {0.f};
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                if (s4 < 2 * (rho + 1)) {            // M is lower triangular: tokens j <= r only
                    wt = __builtin_amdgcn_mfma_f32_32x32x16_f16(gk[s4], mf[rho][s4], wt, 0, 0, 0);
                    u = __builtin_amdgcn_mfma_f32_32x32x16_f16(mf[rho][s4], vv[s4], u, 0, 0, 0);
                }
            }
            // -W: registers 8s..8s+7 of a lane are its 8 contraction slots of K-step s
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4 o4;
#pragma unroll
                for (int z = 0; z < 4; ++z) o4[z] = pack_h2(-wt[8 * s + 2 * z], -wt[8 * s + 2 * z + 1]);
                slot_store16<kPolicy>(out, kOffWn + frag_rts(rho, wave, s) * kFragBytes + lane * 16, o4);
            }
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) {            // U as fp16: kda_scan rounds V_new = U - W S to fp16 anyway
                u32x4 o4;
#pragma unroll
                for (int z = 0; z < 4; ++z) o4[z] = pack_h2(u[8 * j2 + 2 * z], u[8 * j2 + 2 * z + 1]);
                slot_store16<kPolicy>(out, kOffU + (rho * 4 + wave) * kUTileBytes + (j2 * 64 + lane) * 16, o4);
            }
        }
    }
    if (kHandoff) {
        // Hand the finished slot to kda_scan.  Every store to the slot is a write-through store;
        // each wave waits until all of its stores have completed (vmcnt(0): a workgroup barrier
        // alone does not wait for global stores), so after the barrier the slot is in place,
        // device-wide, and one lane raises its flag.
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
        __syncthreads();
        if (tid == 0)
            __hip_atomic_store(ready + ((int64_t)n * H + h) * seg_chunks + cl, epoch, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ----------------------------------------------------------------------------------
// kda_scan
// ----------------------------------------------------------------------------------
// One workgroup of eight waves walks the chunks of one (sequence, head).  Wave (c, p) owns the
// 32-column slice c of the state for the two d_k tiles 2p, 2p+1, and the token tile p of V_new and
// O.  A chunk therefore costs each wave 26-28 MFMAs (32x32x16) instead of 54, at the price of two
// exchanges through LDS per chunk: the fp16 copies of S (every wave needs all four d_k tiles as
// an operand) and of V_new (both token tiles).  All other operands stream from the LDS copy of the
// workspace slot.  The slot of chunk c + 2 is fetched into registers while chunk c computes and
// written to the other LDS stage at the end of chunk c + 1, so a fetch has two full steps to
// arrive.  O is accumulated transposed (operands swapped), so a lane owns four consecutive output
// columns and stores 16 bytes at a time.  Two optional features are compiled in per template
// flag: slots produced by a kda_intra that runs at the same time (kFlags) and the output gate
// (kEpi).
#define KDA_FENCE() __builtin_amdgcn_sched_barrier(0)

namespace scan {
// compile-time loop: f(integral_constant<int, I>) for I in [0, N)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int kUnits = kLdsBlockBytes / 16;                  // 16-byte units per staged block
constexpr int kXS = 2 * kLdsBlockBytes;                      // fp16 S exchange: [c][tau][s] frags
constexpr int kXV = kXS + 4 * 4 * 2 * kFragBytes;            // fp16 V_new exchange: [c][rho][s] frags
constexpr int kRed = kXV + 4 * 2 * 2 * kFragBytes;          // fp32 [2][4][32] sums of squares (output gate)
constexpr int kNormW = kRed + 2 * 4 * 32 * 4;                // fp32 [128] RMSNorm weight (output gate)
constexpr int kLds = kNormW + D * 4;
static_assert(kLds <= 160 * 1024, "kda_scan exceeds the 160 KiB of LDS");

// MFMA slots of wave half P, in issue order:
//   0..7   V_new tile P:  W(P, tau, s),  tau = i / 2, s = i % 2
//   8..15  O^T tile P:    Gamma.Q(P, tau, s)
//   16..23 state tiles 2P, 2P+1: decayed K^T (tau, rho, s): tau = 2P + (j / 4), rho = (j % 4) / 2, s = j % 2
//   24..   O^T tile P += A_qk(P, rho_i, s): rho_i = 0 (and 1 when P = 1)
template <int P> constexpr int num_slots() { return 24 + 2 * (P + 1); }
template <int P> constexpr int slot_lds_offset(int i)
{
    if (i < 8) return kOffWn + frag_rts(P, i / 2, i % 2) * kFragBytes;
    if (i < 16) return kOffQp + frag_rts(P, (i - 8) / 2, (i - 8) % 2) * kFragBytes;
    if (i < 24) {
        const int j = i - 16;
        return kOffKt + frag_trs(2 * P + j / 4, (j % 4) / 2, j % 2) * kFragBytes;
    }
    const int j = i - 24;
    return kOffAqk + frag_aqk(P, j / 2, j % 2) * kFragBytes;
}
}  // namespace scan

// Waits (one lane) until the producer has raised `*flag` to `epoch`.  The wait is bounded: after
// about two seconds the lane records the failure in *status and the kernel runs on with whatever
// the slot holds, so that every wave still reaches the end of the grid.
__device__ __noinline__ void wait_ready(const uint32_t *flag, uint32_t epoch, uint32_t *status, bool &gave_up)
{
    if (gave_up) return;
    const uint64_t t0 = wall_clock64();                     // 100 MHz
    while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) {
        __builtin_amdgcn_s_sleep(8);
        if (wall_clock64() - t0 > 200000000ull) {
            gave_up = true;
            __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
    }
}

// Output gate of Section 4, applied to O before it is stored (kEpi): gate logits [B,T,H,dv] in the
// input dtype, RMSNorm weight [dv] (NULL = ones) and epsilon.  out_bf16 applies with or without the gate.
struct EpiParams {
    const uint16_t *gate;    // caller's gate logits (read by kda_intra, which stages them)
    const float *norm_w;
    float eps;
    int out_bf16;            // o is stored as bf16 (round to nearest even) instead of fp32
    const uint8_t *gate_ws;  // staged gate logits: kGateSlotBytes per slot, same order as the slots
};

// kRole selects what one pass over a range of chunks computes (the time-split scan below):
//   kRoleFull   the scan itself: state from state_in (zero if NULL), outputs written
//   kRoleT      the d_k x d_k transition of the range: starts from the identity, drops U (the
//               recurrence is affine in the state: S_out = T S_in + B), writes no output
//   kRoleB      the offset of the range: starts from zero, keeps U, writes no output
constexpr int kRoleFull = 0, kRoleT = 1, kRoleB = 2;

template <int P, bool kFlags, bool kEpi, int kRole = kRoleFull>
__device__ __forceinline__ void kda_scan_body(uint8_t *lds, const uint8_t *slot0, int64_t slot_stride,
                                              const float *state_in, float *state_out, void *o,
                                              int64_t st_base, int64_t tok_base, int64_t len, int H,
                                              int64_t c_begin, int64_t c_end, int h,
                                              const uint32_t *ready, uint32_t epoch, uint32_t *status,
                                              const EpiParams epi)
{
    using namespace scan;
    constexpr int LA = 6, RING = 8;
    constexpr int NS = num_slots<P>();
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int x = lane & 31, hh = lane >> 5;
    const int c = wave & 3;                                  // column slice of S, V_new, O
    const uint32_t lane16 = (uint32_t)lane * 16;

    // own state tiles in accumulator order: S[t][j] = S(dk = 32 (2P + t) + acc_row(j, hh), dv = 32 c + x)
    f32x16 S[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j)
        {
            const int row = 32 * (2 * P + t) + acc_row(j, hh);
            if (kRole == kRoleT)      S[t][j] = (row == 32 * (wave & 3) + (lane & 31)) ? 1.f : 0.f;
            else if (kRole == kRoleB) S[t][j] = 0.f;
            else                      S[t][j] = state_in ? state_in[st_base + (int64_t)row * D] : 0.f;
        }

    if (c_begin < c_end) {
        // Workspace slot -> LDS: the block of chunk ci is fetched into registers two steps ahead
        // (register set ci % 2), written to LDS stage ci % 2 at the end of step ci - 1 and read in
        // step ci, so that a fetch has two full steps to complete.  Thread tid moves the 16-byte
        // units tid, tid + 512, ...; the wave's U tile (P, c) travels the same way.
        constexpr int kMyUnits = (kUnits + 511) / 512;
        const uint32_t u_src = (uint32_t)(kOffU + (P * 4 + c) * kUTileBytes) + lane16;   // U tile (P, c): 2 x 1 KiB
        u32x4 pre[2][kMyUnits];
        u32x4 un[2][2];
        u32x4 gt[2][2];                                      // kEpi: the wave's tile of staged gate logits
        const int64_t gate_stride = (int64_t)H * kGateSlotBytes;
        // The transition and offset passes of the time-split scan write no output: they leave
        // Gamma.Q (units 1024 .. 2047: i = 2, 3) and A_qk (the units of i = 6 below gamma^C) where
        // they are, and the transition pass U as well.
        static_assert(kOffQp == 2 * 512 * 16 && kOffKt == 4 * 512 * 16 && kOffAqk == 6 * 512 * 16, "unit ranges of the skipped operands");
        auto wanted = [&](const int i, const int unit) __attribute__((always_inline)) {
            return kRole == kRoleFull || !(i == 2 || i == 3 || (i == 6 && unit * 16 < kOffGc));
        };
        auto fetch = [&](const int64_t rel, u32x4 *blk, u32x4 *u, u32x4 *g) __attribute__((always_inline)) {
            const uint8_t *src = slot0 + rel * slot_stride;
            const __amdgpu_buffer_rsrc_t rs = slot_resource(src);
            if (kEpi) {
                const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<uint8_t *>(epi.gate_ws + rel * gate_stride), 0, kGateSlotBytes, 0x00020000);
                const int goff = (P * 4 + c) * kGateTileBytes + (int)lane16;
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    g[i] = kFlags ? slot_load16<kCacheDevice>(rg, goff + i * 1024) : slot_load16<0>(rg, goff + i * 1024);
            }
            // (kFlags: the slot was written while this kernel runs, hence device-scope loads)
            constexpr int kPol = kFlags ? kCacheDevice : 0;
#pragma unroll
            for (int i = 0; i < kMyUnits; ++i) {
                const int unit = tid + i * 512;
                if (unit < kUnits && wanted(i, unit)) blk[i] = slot_load16<kPol>(rs, unit * 16);
            }
            if (kRole != kRoleT) {
#pragma unroll
                for (int i = 0; i < 2; ++i) u[i] = slot_load16<kPol>(rs, (int)u_src + i * 1024);
            }
        };
        auto publish = [&](const u32x4 *blk, int stage) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < kMyUnits; ++i) {
                const int unit = tid + i * 512;
                if (unit < kUnits && wanted(i, unit))
                    *reinterpret_cast<u32x4 *>(lds + stage * kLdsBlockBytes + unit * 16) = blk[i];
            }
        };
        // With kFlags the slots are produced while this kernel runs: lane 0 of the workgroup
        // checks the flag of chunk ci + 2 before the barrier that precedes its fetch; the flag is
        // read one step early (`seen`), so the check normally costs nothing.
        const bool poll = kFlags && (P == 0) && tid == 0;
        bool gave_up = false;
        uint32_t seen = epoch;
        if (kFlags) {
            if (poll) {
                wait_ready(ready, epoch, status, gave_up);
                if (c_begin + 1 < c_end) wait_ready(ready + 1, epoch, status, gave_up);
            }
            __syncthreads();
        }
        // (the flag load goes out before the slot loads: loads return in order, so the check of
        // `seen` one step later must not have to wait for a whole slot fetch that was issued first)
        if (kFlags) {
            const int64_t cf = (c_begin + 2 < c_end) ? 2 : c_end - 1 - c_begin;
            seen = __hip_atomic_load(ready + cf, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        fetch(0, pre[0], un[0], gt[0]);
        if (c_begin + 1 < c_end) fetch(1, pre[1], un[1], gt[1]);
        publish(pre[0], 0);

        const uint32_t o_rstride = (uint32_t)H * D * 4;      // bytes between consecutive tokens of o
        // O^T accumulator: lane (token 32 P + x, hh), registers 4q..4q+3 = columns 32 c + 8 q + 4 hh + 0..3
        const uint32_t o_lane = (uint32_t)(32 * P + x) * o_rstride + (uint32_t)(32 * c + 4 * hh) * 4;
        uint8_t *xs = lds + kXS + c * (4 * 2 * kFragBytes) + lane16;    // + (tau * 2 + s) * kFragBytes
        uint8_t *xv = lds + kXV + c * (2 * 2 * kFragBytes) + lane16;    // + (rho * 2 + s) * kFragBytes

        // one chunk; `stage` (compile-time parity) is its LDS stage and register set
        auto chunk_step = [&](const int64_t ci, auto stage_c) __attribute__((always_inline)) {
            constexpr int stage = decltype(stage_c)::value;
            const uint8_t *cur = lds + stage * kLdsBlockBytes + lane16;
            const float *gc = reinterpret_cast<const float *>(lds + stage * kLdsBlockBytes + kOffGc) + 4 * hh;
            const bool more = ci + 1 < c_end;

            // ---- publish the fp16 copy of the own state tiles ----
            h8 Sb[4][2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) Sb[2 * P + t][s][e] = (_Float16)S[t][8 * s + e];
                    *reinterpret_cast<h8 *>(xs + ((2 * P + t) * 2 + s) * kFragBytes) = Sb[2 * P + t][s];
                }
            if (poll && ci + 2 < c_end && seen != epoch)
                wait_ready(ready + (ci + 2 - c_begin), epoch, status, gave_up);
            __syncthreads();                                                 // B1: S exchange and LDS stage ready

            f32x16 av, ao = {0.f};
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int z = 0; z < 4; ++z) {
                    const uint32_t w2 = un[stage][i][z];     // (a copy first: bit_cast straight from a vector element misreads it)
                    const h2 pr = __builtin_bit_cast(h2, w2);
                    av[8 * i + 2 * z] = (kRole == kRoleT) ? 0.f : (float)pr[0];
                    av[8 * i + 2 * z + 1] = (kRole == kRoleT) ? 0.f : (float)pr[1];
                }
            // this register set is free now: start fetching chunk ci + 2 into it
            // kEpi: this chunk's gate logits leave their register set before it is refilled;
            // gate_raw[q4][w] = columns 8 q4 + 4 hh + 2 w, + 1
            uint32_t gate_raw[4][2];
            if (kEpi) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                    for (int w = 0; w < 2; ++w) gate_raw[q4][w] = gt[stage][q4 / 2][(q4 % 2) * 2 + w];
            }
            // (every lane loads the flag, unconditionally and past the end clamped to the last chunk:
            // a fixed number of loads in flight lets the check wait for exactly this one)
            if (kFlags) {
                const int64_t cf = (ci + 3 < c_end) ? ci + 3 : c_end - 1;
                seen = __hip_atomic_load(ready + (cf - c_begin), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            // (issued unconditionally, past the end the last slot is simply fetched again: with a
            // fixed number of loads in flight behind them, earlier loads can be waited for one by one)
            {
                const int64_t cf = (ci + 2 < c_end) ? ci + 2 : c_end - 1;
                fetch(cf - c_begin, pre[stage], un[stage], gt[stage]);
            }
            // the partner's two d_k tiles of S
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    Sb[2 * (1 - P) + t][s] = *reinterpret_cast<const h8 *>(xs + ((2 * (1 - P) + t) * 2 + s) * kFragBytes);

            h8 ring[RING];
            h8 Vb[2][2];
#pragma unroll
            for (int i = 0; i < LA; ++i)
                ring[i % RING] = *reinterpret_cast<const h8 *>(cur + slot_lds_offset<P>(i));

            float sg[16];                                    // kEpi: Sigmoid(gate) * norm weight per output
            static_for<0, NS>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value;
                if constexpr (kEpi && i >= 16 && i < 24) {
                    // two gate factors per MFMA slot: the transcendentals run under the matrix cores
                    constexpr int j = i - 16, q4 = j / 2, w = j % 2;
                    float g0, g1;
                    unpack_bf16x2(gate_raw[q4][w], g0, g1);
                    const float2 nw = *reinterpret_cast<const float2 *>(lds + kNormW + (32 * c + 4 * hh + 8 * q4 + 2 * w) * 4);
                    sg[4 * q4 + 2 * w] = nw.x * __builtin_amdgcn_rcpf(1.f + fast_exp2(-g0 * kLog2e));
                    sg[4 * q4 + 2 * w + 1] = nw.y * __builtin_amdgcn_rcpf(1.f + fast_exp2(-g1 * kLog2e));
                }
                if constexpr (i + LA < NS && (kRole == kRoleFull || !((i + LA >= 8 && i + LA < 16) || i + LA >= 24)))
                    ring[(i + LA) % RING] = *reinterpret_cast<const h8 *>(cur + slot_lds_offset<P>(i + LA));
                const h8 a = ring[i % RING];
                if constexpr (i < 8) {
                    // V_new = U + (-W) S
                    av = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Sb[i / 2][i % 2], av, 0, 0, 0);
                    if constexpr (i == 7) {
                        // publish the fp16 copy of the own token tile of V_new
#pragma unroll
                        for (int s = 0; s < 2; ++s) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) Vb[P][s][e] = (_Float16)av[8 * s + e];
                            *reinterpret_cast<h8 *>(xv + (P * 2 + s) * kFragBytes) = Vb[P][s];
                        }
                    }
                } else if constexpr (i < 16) {
                    // O^T = S^T (Gamma.Q)^T
                    if constexpr (kRole == kRoleFull)
                        ao = __builtin_amdgcn_mfma_f32_32x32x16_f16(Sb[(i - 8) / 2][(i - 8) % 2], a, ao, 0, 0, 0);
                    if constexpr (i == 10 || i == 12) {
                        // S <- Diag(gamma^C) S on the own tiles (their fp16 copies are taken)
                        constexpr int t = (i - 10) / 2;
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const f32x4 gv = *reinterpret_cast<const f32x4 *>(gc + 32 * (2 * P + t) + 8 * q4);
#pragma unroll
                            for (int z = 0; z < 4; ++z) S[t][4 * q4 + z] *= gv[z];
                        }
                    }
                    if constexpr (i == 15) {
                        __syncthreads();                                         // B2: V_new exchange complete
#pragma unroll
                        for (int s = 0; s < 2; ++s)
                            Vb[1 - P][s] = *reinterpret_cast<const h8 *>(xv + ((1 - P) * 2 + s) * kFragBytes);
                    }
                } else if constexpr (i < 24) {
                    // S += (Gamma^{i->C}.K)^T V_new on the own d_k tiles
                    constexpr int j = i - 16;
                    S[j / 4] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, Vb[(j % 4) / 2][j % 2], S[j / 4], 0, 0, 0);
                } else {
                    // O^T += V_new^T Tril(A_qk)^T
                    constexpr int j = i - 24;
                    if constexpr (kRole == kRoleFull)
                        ao = __builtin_amdgcn_mfma_f32_32x32x16_f16(Vb[j / 2][j % 2], a, ao, 0, 0, 0);
                }
                KDA_FENCE();   // keeps each operand read LA slots ahead of its MFMA
            });

            if (kEpi) {
                // O <- Sigmoid(gate) * RMSNorm(O) * w.  A token's 128 outputs sit in the four waves
                // of this token tile: lane-local sum of squares, the two lane halves by a swap,
                // the four waves through LDS.
                float ssq = 0.f;
#pragma unroll
                for (int j = 0; j < 16; ++j) ssq = fmaf(ao[j], ao[j], ssq);
                ssq += __shfl_xor(ssq, 32);
                float *red = reinterpret_cast<float *>(lds + kRed);
                if (hh == 0) red[(P * 4 + c) * 32 + x] = ssq;
                // the next chunk's block goes to the other LDS stage while the partial sums gather
                if (more) publish(pre[stage ^ 1], stage ^ 1);
                __syncthreads();                                             // B3 (kEpi only)
                const float tot = red[(P * 4 + 0) * 32 + x] + red[(P * 4 + 1) * 32 + x] +
                                  red[(P * 4 + 2) * 32 + x] + red[(P * 4 + 3) * 32 + x];
                const float rstd = __builtin_amdgcn_rsqf(tot * (1.0f / D) + epi.eps);
#pragma unroll
                for (int j = 0; j < 16; ++j) ao[j] *= rstd * sg[j];
            }
            // write O (already scaled): 16 bytes per store
            if (kRole == kRoleFull) {
                const int64_t t0 = ci * kChunk;
                if (!epi.out_bf16) {
                    uint8_t *obase = static_cast<uint8_t *>(o) + ((tok_base + t0) * H + h) * (int64_t)(D * 4);
                    if (t0 + 32 * P + x < len) {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            f32x4 val = {ao[4 * q4], ao[4 * q4 + 1], ao[4 * q4 + 2], ao[4 * q4 + 3]};
                            *reinterpret_cast<f32x4 *>(obase + (o_lane + 32 * q4)) = val;
                        }
                    }
                } else {
                    // bf16: w[2 q4 + z] = columns 8 q4 + 4 hh + 2 z, + 1.  The two lanes of a token
                    // trade halves (lanes 0-31 hand over q4 = 2, 3 and receive the partner's q4 = 0, 1),
                    // so each lane ends up with two runs of eight consecutive columns: two stores
                    // instead of four.
                    uint32_t w[8];
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        w[2 * q4] = pack_bf16x2(ao[4 * q4], ao[4 * q4 + 1]);
                        w[2 * q4 + 1] = pack_bf16x2(ao[4 * q4 + 2], ao[4 * q4 + 3]);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(w[i], w[4 + i], false, false);
                        w[i] = sw[0]; w[4 + i] = sw[1];
                    }
                    uint8_t *obase = static_cast<uint8_t *>(o) + ((tok_base + t0) * H + h) * (int64_t)(D * 2);
                    if (t0 + 32 * P + x < len) {
#pragma unroll
                        for (int qq = 0; qq < 2; ++qq) {
                            u32x4 val = {w[2 * qq], w[2 * qq + 1], w[4 + 2 * qq], w[4 + 2 * qq + 1]};
                            *reinterpret_cast<u32x4 *>(obase + (uint32_t)(32 * P + x) * (o_rstride / 2) +
                                                       (uint32_t)(32 * c + 8 * (qq + 2 * hh)) * 2) = val;
                        }
                    }
                }
            }
            KDA_FENCE();
            // the next chunk's block (fetched one step ago) goes to the other LDS stage
            if (!kEpi && more) publish(pre[stage ^ 1], stage ^ 1);
        };
        for (int64_t ci = c_begin; ci < c_end; ci += 2) {
            chunk_step(ci, std::integral_constant<int, 0>{});
            if (ci + 1 < c_end) chunk_step(ci + 1, std::integral_constant<int, 1>{});
        }
    }

    if (state_out && (state_out != state_in || c_begin < c_end)) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                state_out[st_base + (int64_t)(32 * (2 * P + t) + acc_row(j, hh)) * D] = S[t][j];
    }
}

// kFlags: the slots are produced by a kda_intra that runs at the same time (per-slot ready flags).
template <bool kFlags, bool kEpi>
__global__ __launch_bounds__(512)
void kda_scan_kernel(const uint8_t *__restrict__ ws, const float *state_in, float *state_out,
                     const int32_t *__restrict__ cu_seqlens, void *__restrict__ o, int64_t T, int H,
                     int64_t seg_chunks, int64_t seg_index, const uint32_t *ready, uint32_t epoch,
                     uint32_t *status, EpiParams epi)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x / H, h = blockIdx.x % H;

    int64_t tok_base, len;
    if (cu_seqlens) { tok_base = cu_seqlens[n]; len = (int64_t)cu_seqlens[n + 1] - tok_base; }
    else            { tok_base = (int64_t)n * T; len = T; }
    const int64_t nchunks = (len + kChunk - 1) / kChunk;
    const int64_t c_begin = seg_index * seg_chunks;
    const int64_t c_end = (nchunks < c_begin + seg_chunks) ? nchunks : c_begin + seg_chunks;
    const int64_t st_base = ((int64_t)n * H + h) * (int64_t)(D * D) + 32 * (wave & 3) + (lane & 31);
    const uint8_t *slot0 = ws + (((int64_t)n * seg_chunks) * H + h) * (int64_t)kSlotBytes;
    const int64_t slot_stride = (int64_t)H * kSlotBytes;

    if (kEpi && threadIdx.x < D)     // RMSNorm weights: read by every step after its first barrier
        reinterpret_cast<float *>(lds + scan::kNormW)[threadIdx.x] = epi.norm_w ? epi.norm_w[threadIdx.x] : 1.f;
    const uint32_t *flag0 = kFlags ? ready + (int64_t)blockIdx.x * seg_chunks : nullptr;
    // nothing is waited for without flags: leave a clean status word for kda_chunk_fwd_check
    if (!kFlags && status && blockIdx.x == 0 && threadIdx.x == 0) *status = 0;

    if (kEpi) epi.gate_ws += (((int64_t)n * seg_chunks) * H + h) * (int64_t)kGateSlotBytes;   // this pair's first slot
    if (wave < 4)
        kda_scan_body<0, kFlags, kEpi>(lds, slot0, slot_stride, state_in, state_out, o, st_base, tok_base, len, H,
                                       c_begin, c_end, h, flag0, epoch, status, epi);
    else
        kda_scan_body<1, kFlags, kEpi>(lds, slot0, slot_stride, state_in, state_out, o, st_base, tok_base, len, H,
                                       c_begin, c_end, h, flag0, epoch, status, epi);
}

// Time-split scan for few (sequence, head) pairs: the chunk axis is cut into `parts` ranges, the
// first of `part0_len` chunk indices and the others of `part_len` (the first range is walked by the
// full scan, which is slower per step than the transition and offset passes of the other ranges,
// so it is made shorter), and 2 parts - 3 workgroups work on one pair side by side, in one launch.
//   blockIdx.y = 0              scans range 0 from h0 (outputs and all) and leaves its final state
//                               in E[0]; later it scans the last range from E[parts - 2] and
//                               delivers the final state.
//   blockIdx.y = 2 p - 1        computes the transition T_p of range p = 1 .. parts - 2; later it
//                               scans range p from E[p - 1].
//   blockIdx.y = 2 p            computes the offset B_p of range p.
// Between the phases, workgroups blockIdx.y = 1 .. workers form E[p] = T_p E[p-1] + B_p for
// p = 1 .. parts - 2, each on its own slice of the d_v columns (the columns do not interact).
// Results travel through the workspace (E, Tm, Bm: arrays of [pairs][128][128] fp32 states, one
// per range) under per-pair counters: pf[p] = slices of E[p] that are complete (E[0]: set to
// `workers` at once), pf[8 + p] / pf[16 + p] = T_p / B_p complete.  Every producer makes its stores
// visible with a device-scope release before it raises the counter, every consumer follows its
// (bounded) wait with a device-scope acquire.  No first-phase work waits for anything and a
// launch has fewer workgroups than half the compute units, so every wait ends.
constexpr int kSplitFlagsPerPair = 24;

// E[p][:, col0 .. col0 + 16 CW) for p = 1 .. parts - 2, in fp32, by one 512-thread workgroup.
// Thread (ty, tx) owns rows 4 ty .. 4 ty + 3 and columns col0 + CW tx .. + CW - 1; the current
// slice of E sits in LDS.  All T_p and B_p are awaited first (they finish before E[0] does) and
// pulled into this die's L2; after that the chain crosses no fence: E[0] is read and E[p] written
// with device-scope accesses.
template <int CW>
__device__ __forceinline__ void kda_fold_slices(float *sE, float *E, const float *Tm, const float *Bm,
                                                int64_t pair_states, int64_t pair_base, int col0, int parts,
                                                int workers, uint32_t *pf, uint32_t *status, bool &gave_up)
{
    constexpr int NC = 16 * CW;
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    if (tid == 0)
        for (int p = 1; p <= parts - 2; ++p) {
            wait_ready(pf + 8 + p, 1u, status, gave_up);
            wait_ready(pf + 16 + p, 1u, status, gave_up);
        }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    {
        f32x4 touch = {0.f, 0.f, 0.f, 0.f};
        for (int p = 1; p <= parts - 2; ++p)
            for (int i = tid; i < D * D / 4; i += 512)
                touch += *reinterpret_cast<const f32x4 *>(Tm + p * pair_states + pair_base + 4 * i);
        asm volatile("" ::"v"(touch));
    }
    if (tid == 0) wait_ready(pf, (uint32_t)workers, status, gave_up);
    __syncthreads();
    for (int i = tid; i < D * NC; i += 512)
        sE[i] = __hip_atomic_load(E + pair_base + (int64_t)(i / NC) * D + col0 + (i % NC), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    for (int p = 1; p <= parts - 2; ++p) {
        const float *Tp = Tm + p * pair_states + pair_base;
        const float *Bp = Bm + p * pair_states + pair_base + col0 + CW * tx;
        float acc[4][CW];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int z = 0; z < CW; ++z) acc[i][z] = Bp[(int64_t)(4 * ty + i) * D + z];
        for (int k4 = 0; k4 < D / 4; ++k4) {
            f32x4 a[4];
            float b[4][CW];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const f32x4 *>(Tp + (int64_t)(4 * ty + i) * D + 4 * k4);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int z = 0; z < CW; ++z) b[kk][z] = sE[(4 * k4 + kk) * NC + CW * tx + z];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int z = 0; z < CW; ++z) acc[i][z] = fmaf(a[i][kk], b[kk][z], acc[i][z]);
        }
        __syncthreads();                                     // every thread is done reading the old slice
        float *Ep = E + p * pair_states + pair_base + col0 + CW * tx;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int z = 0; z < CW; ++z) {
                sE[(4 * ty + i) * NC + CW * tx + z] = acc[i][z];
                __hip_atomic_store(Ep + (int64_t)(4 * ty + i) * D + z, acc[i][z], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): the write-through stores have landed
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(pf + p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <bool kFlags, bool kEpi>
__global__ __launch_bounds__(512)
void kda_scan_split_kernel(const uint8_t *__restrict__ ws, const float *h0, float *E, float *Tm, float *Bm,
                           float *state_final, const int32_t *__restrict__ cu_seqlens, void *__restrict__ o,
                           int64_t T, int H, int64_t seg_chunks, int64_t seg_index, int64_t part_len,
                           int64_t part0_len, int parts, const uint32_t *ready, uint32_t epoch, uint32_t *status,
                           uint32_t *split_flags, EpiParams epi)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x / H, h = blockIdx.x % H;
    const int64_t pair_states = (int64_t)gridDim.x * (D * D);
    const int64_t pair_base = (int64_t)blockIdx.x * (D * D);

    int64_t tok_base, len;
    if (cu_seqlens) { tok_base = cu_seqlens[n]; len = (int64_t)cu_seqlens[n + 1] - tok_base; }
    else            { tok_base = (int64_t)n * T; len = T; }
    // chunk indices below are local to the time segment [cbase, cbase + seg_chunks) of this launch
    const int64_t cbase = seg_index * seg_chunks;
    int64_t nchunks = (len + kChunk - 1) / kChunk - cbase;
    if (nchunks < 0) nchunks = 0;
    if (nchunks > seg_chunks) nchunks = seg_chunks;

    const int y = (int)blockIdx.y;
    const int kind = (y == 0) ? kRoleFull : ((y & 1) ? kRoleT : kRoleB);
    const int mid = (y + 1) / 2;                              // the range of the first phase
    const int workers = (parts - 2 >= 4) ? 8 : (parts - 2 >= 2) ? 4 : 2;   // among the 2 parts - 4 others
    uint32_t *pf = split_flags + (int64_t)blockIdx.x * kSplitFlagsPerPair;
    bool gave_up = false;

    const int64_t st_base = pair_base + 32 * (wave & 3) + (lane & 31);
    const int64_t slot_stride = (int64_t)H * kSlotBytes;
    if (kEpi && threadIdx.x < D)     // RMSNorm weights of the output gate (beyond what the fold uses of the LDS)
        reinterpret_cast<float *>(lds + scan::kNormW)[threadIdx.x] = epi.norm_w ? epi.norm_w[threadIdx.x] : 1.f;
    const uint8_t *gate_base = epi.gate_ws;

    // (the output gate concerns the full scan only; the passes without output ignore it)
#define KDA_SCAN_PART(ROLE, EPI)                                                                                  \
    if (EPI) epi.gate_ws = gate_base + (((int64_t)n * seg_chunks + c_begin) * H + h) * (int64_t)kGateSlotBytes;   \
    if (wave < 4)                                                                                                 \
        kda_scan_body<0, kFlags, EPI, ROLE>(lds, slot0, slot_stride, state_in, state_out, o, st_base, tok_base,   \
                                            len, H, cbase + c_begin, cbase + c_end, h, flag0, epoch, status, epi); \
    else                                                                                                          \
        kda_scan_body<1, kFlags, EPI, ROLE>(lds, slot0, slot_stride, state_in, state_out, o, st_base, tok_base,   \
                                            len, H, cbase + c_begin, cbase + c_end, h, flag0, epoch, status, epi)
    {   // first phase: the own range, from h0 / the identity / zero
        const float *state_in = (y == 0) ? h0 : nullptr;
        float *state_out = (y == 0) ? E : (kind == kRoleT ? Tm : Bm) + mid * pair_states;
        int64_t c_begin = (mid == 0) ? 0 : part0_len + (mid - 1) * part_len;
        int64_t c_end = c_begin + ((mid == 0) ? part0_len : part_len);
        if (c_begin > nchunks) c_begin = nchunks;
        if (c_end > nchunks) c_end = nchunks;
        const uint8_t *slot0 = ws + (((int64_t)n * seg_chunks + c_begin) * H + h) * (int64_t)kSlotBytes;
        const uint32_t *flag0 = kFlags ? ready + (int64_t)blockIdx.x * seg_chunks + c_begin : nullptr;
        if (kind == kRoleFull) { KDA_SCAN_PART(kRoleFull, kEpi); }
        else if (kind == kRoleT) { KDA_SCAN_PART(kRoleT, false); }
        else { KDA_SCAN_PART(kRoleB, false); }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t *f = (kind == kRoleFull) ? pf : (kind == kRoleT) ? pf + 8 + mid : pf + 16 + mid;
            __hip_atomic_store(f, (kind == kRoleFull) ? (uint32_t)workers : 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (y >= 1 && y <= workers) {
        float *sE = reinterpret_cast<float *>(lds);
        const int w = y - 1;
        if (workers == 8)      kda_fold_slices<1>(sE, E, Tm, Bm, pair_states, pair_base, 16 * w, parts, workers, pf, status, gave_up);
        else if (workers == 4) kda_fold_slices<2>(sE, E, Tm, Bm, pair_states, pair_base, 32 * w, parts, workers, pf, status, gave_up);
        else                   kda_fold_slices<4>(sE, E, Tm, Bm, pair_states, pair_base, 64 * w, parts, workers, pf, status, gave_up);
    }
    if (kind == kRoleB) return;
    {   // second phase: the scan of a range whose initial state is now known
        const int part = (y == 0) ? parts - 1 : mid;
        const float *state_in = E + (part - 1) * pair_states;
        float *state_out = (y == 0) ? state_final : nullptr;
        if (threadIdx.x == 0) wait_ready(pf + part - 1, (uint32_t)workers, status, gave_up);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        int64_t c_begin = part0_len + (part - 1) * part_len, c_end = c_begin + part_len;   // part >= 1 here
        if (c_begin > nchunks) c_begin = nchunks;
        if (c_end > nchunks) c_end = nchunks;
        const uint8_t *slot0 = ws + (((int64_t)n * seg_chunks + c_begin) * H + h) * (int64_t)kSlotBytes;
        const uint32_t *flag0 = kFlags ? ready + (int64_t)blockIdx.x * seg_chunks + c_begin : nullptr;
        KDA_SCAN_PART(kRoleFull, kEpi);
    }
#undef KDA_SCAN_PART
}

// flags and status word of the overlapped mode start every call at zero
__global__ void kda_fill_u32_kernel(uint32_t *p, int64_t n, uint32_t value, uint32_t *one_more)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
    if (i == 0) *one_more = value;
}

// ----------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------
static int64_t max_chunks_per_seq(const kda_dims *d)
{
    int64_t longest = d->seqlen;
    if (d->num_seqs != d->batch || d->batch == 1) {           // packed (or a single row)
        if (d->max_seqlen > 0 && d->max_seqlen < longest) longest = d->max_seqlen;
    }
    return (longest + kChunk - 1) / kChunk;
}

static size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace: [status word, 256 B][slots of one segment][state carry][ready flags, one per slot]
// [time-split counters and states][staged gate logits]; the last two only when the call can use them.
static SegPlan plan_with(const kda_dims *d, int64_t sc, bool gate)
{
    SegPlan p;
    const int64_t maxc = max_chunks_per_seq(d);
    const size_t streams = (size_t)d->num_seqs * d->heads;
    const size_t carry = streams * D * D * sizeof(float);
    p.seg_chunks = sc;
    p.num_segments = (maxc + sc - 1) / sc;
    p.status_offset = 0;                                  // the same place whatever the segment size
    p.slots_offset = 256;
    p.carry_offset = p.slots_offset + (size_t)sc * streams * kSlotBytes;
    p.flags_offset = p.carry_offset + carry;
    p.split_offset = round_up(p.flags_offset + (size_t)sc * streams * sizeof(uint32_t), 256);
    // counters and states of the time-split scan, when the call qualifies for it
    const bool split = streams <= (size_t)kSplitMaxPairs && sc >= kSplitMinChunks;
    p.total_bytes = p.split_offset + (split ? kSplitFlagBytes + 3 * (size_t)kSplitMaxParts * carry : 0);
    p.gate_offset = 0;
    if (gate) {
        p.gate_offset = round_up(p.total_bytes, 256);
        p.total_bytes = p.gate_offset + (size_t)sc * streams * kGateSlotBytes;
    }
    return p;
}

// Number of ranges for the time-split scan (1 = plain scan).  The launch keeps 2 parts - 3 compute
// units per pair busy; it gets at most three eighths of the device, so that kda_intra, which runs
// beside it and is the larger half of the work, keeps the rest (measured on 2 to 40 pairs: beyond
// that limit the plain scan wins).  Among the admissible numbers the one with the smallest
// estimated duration is taken, the plain scan included.  The estimate (microseconds; constants
// measured on MI355X): a step of the scan 2.85, a chunk of kda_intra 9.5 on one compute unit, the
// fold and the extra start-up of a split launch 60 + 12 per middle range.  The first phase needs
// the first parts - 1 ranges produced, the last range one more phase after everything before it.
// forced = 3..8: the largest admissible number up to `forced`, whatever the estimate says.
static int split_parts(const SegPlan &plan, const kda_dims *d, int cus, int forced, double *first_ratio)
{
    *first_ratio = 1.0;
    int64_t maxc = max_chunks_per_seq(d);                    // chunks one launch walks
    if (maxc > plan.seg_chunks) maxc = plan.seg_chunks;
    const int64_t pairs = (int64_t)d->num_seqs * d->heads;
    if (pairs > kSplitMaxPairs || maxc < kSplitMinChunks || pairs >= cus) return 1;
    const double step = 2.85, item = 9.5;
    const double items = (double)pairs * (double)maxc;
    const double t_scan = (double)maxc * step, t_intra1 = items * item / (double)(cus - pairs);
    double best = t_scan > t_intra1 ? t_scan : t_intra1;
    int parts = 1;
    for (int p = 3; p <= kSplitMaxParts; ++p) {
        const int64_t len = (maxc + p - 1) / p;
        if (pairs * (2 * p - 3) * 8 > (int64_t)cus * 3 || len < 8) continue;
        const double phase = (double)len * step;
        const double t_intra = items * item / (double)(cus - pairs * (2 * p - 3));
        const double fed = t_intra * (double)(p - 1) / (double)p;
        // The first range is walked by the full scan, the others by passes that write no output and
        // fetch less, about 0.7 of its time per step: when the scan, not kda_intra, sets the pace
        // of the first phase, the first range is made shorter by that ratio (measured: 7-9 % on 2
        // and 4 pairs; a loss where kda_intra is the bound, because the other ranges grow).
        const double ratio = (phase >= 1.5 * fed) ? 0.7 : 1.0;
        if (forced >= 3) {
            if (p <= forced) { parts = p; *first_ratio = ratio; }
            continue;
        }
        const double t1 = phase > fed ? phase : fed;
        double t = t1 + 60.0 + 12.0 * (p - 2) + phase;
        if (t_intra + 2 * step > t) t = t_intra + 2 * step;
        if (t < best) { best = t; parts = p; *first_ratio = ratio; }
    }
    return parts;
}

// The plan with the most chunk indices per segment that fits `workspace_bytes` (full: no limit).
static SegPlan make_plan(const kda_dims *d, size_t workspace_bytes, bool full, bool gate)
{
    const int64_t maxc = max_chunks_per_seq(d);
    int64_t sc = maxc < 1 ? 1 : maxc;
    if (sc > 65535) sc = 65535;                               // grid dimension limit of kda_intra
    if (!full) {
        const size_t streams = (size_t)d->num_seqs * d->heads;
        const size_t per_chunk_index = streams * (kSlotBytes + sizeof(uint32_t) + (gate ? kGateSlotBytes : 0));
        const size_t fixed = plan_with(d, 1, gate).total_bytes - per_chunk_index;
        const size_t avail = workspace_bytes > fixed ? workspace_bytes - fixed : 0;
        const int64_t fit = per_chunk_index ? (int64_t)(avail / per_chunk_index) : sc;
        if (fit < sc) sc = fit;
        if (sc < 1) sc = 1;
        while (sc > 1 && plan_with(d, sc, gate).total_bytes > workspace_bytes) --sc;   // rounding of the flag area
    }
    return plan_with(d, sc, gate);
}

// Raises the dynamic-LDS limit of the prefill kernels, once per device.
static bool reserve_lds()
{
    constexpr int kMaxDevices = 64;
    static bool done[kMaxDevices];                          // same outcome from every thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (done[dev]) return true;
    const int scan_lds = scan::kLds;
    const bool ok =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<false, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<true, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<false, false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_kernel<true, false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_kernel<false, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_kernel<true, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_kernel<false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_kernel<true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_split_kernel<false, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_split_kernel<true, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_split_kernel<false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_split_kernel<true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan_lds) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    done[dev] = ok;
    return ok;
}

// Helper streams and events of the overlapped mode, created on first use, one set per device, never
// destroyed.  Both kernels of an overlapped call run on library streams (kda_scan on `scan`,
// kda_intra on `intra`) that were seen to run at the same time when they were created; the caller's
// stream only carries the events around them, so its own hardware queue does not matter.
struct SideStream {
    hipStream_t stream = nullptr;           // kda_intra
    hipStream_t scan_stream = nullptr;      // kda_scan
    hipEvent_t fork = nullptr, fork_intra = nullptr, join = nullptr, join_scan = nullptr;
    bool tried = false, ok = false;
};

// A hardware queue runs its kernels in order and a process has few of them for all its streams:
// two streams on one queue never overlap.  The probe: a one-thread kernel on `a` polls a device word,
// for a few milliseconds at most, that a kernel on `b` sets.
__device__ uint32_t g_probe_word[2];        // [0] the word, [1] what the polling kernel saw

__global__ void kda_probe_reset_kernel() { g_probe_word[0] = 0u; g_probe_word[1] = 0u; }

__global__ void kda_probe_set_kernel() { __hip_atomic_store(&g_probe_word[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__global__ void kda_probe_poll_kernel()
{
    uint32_t seen = 0u;
    for (int it = 0; it < 4000 && !seen; ++it) {            // bounded: about 4 ms
        seen = __hip_atomic_load(&g_probe_word[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_sleep(32);
    }
    g_probe_word[1] = seen;
}

// The same question for a caller's stream against the kda_intra stream, asked without waiting for
// the caller's stream: the polling kernel goes onto the caller's stream first, then the setting one
// onto the helper stream (on a shared queue the second cannot run before the first has finished),
// the answer is copied to pinned host memory behind the polling kernel and read by a later call.
constexpr int kCallerSlots = 16;
__device__ uint32_t g_caller_probe[kCallerSlots][2];    // [slot][0] the word, [1] what the polling kernel saw

__global__ void kda_caller_set_kernel(int slot, uint32_t token)
{
    __hip_atomic_store(&g_caller_probe[slot][0], token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void kda_caller_poll_kernel(int slot, uint32_t token)
{
    uint32_t seen = 0u;
    for (int it = 0; it < 4000 && seen != token; ++it) {    // bounded: about 4 ms
        seen = __hip_atomic_load(&g_caller_probe[slot][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_sleep(32);
    }
    g_caller_probe[slot][1] = seen;
}

static bool streams_run_together(hipStream_t a, hipStream_t b)
{
    uint32_t seen = 0u;
    hipLaunchKernelGGL(kda_probe_reset_kernel, dim3(1), dim3(1), 0, a);
    if (hipStreamSynchronize(a) != hipSuccess) { (void)hipGetLastError(); return false; }
    hipLaunchKernelGGL(kda_probe_poll_kernel, dim3(1), dim3(1), 0, a);
    hipLaunchKernelGGL(kda_probe_set_kernel, dim3(1), dim3(1), 0, b);
    if (hipStreamSynchronize(b) != hipSuccess || hipStreamSynchronize(a) != hipSuccess ||
        hipMemcpyFromSymbol(&seen, HIP_SYMBOL(g_probe_word), sizeof(seen), sizeof(uint32_t),
                            hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return seen == 1u;
}

// Compute units of the current device (cached per device), 0 on failure.
static int compute_units()
{
    constexpr int kMaxDevices = 64;
    static int table[kMaxDevices];                          // 0 = not asked yet; same value from every thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    if (table[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) { n = 0; (void)hipGetLastError(); }
        table[dev] = n;
    }
    return table[dev];
}

// All overlapped calls of a process share one pair of helper streams per device, and a mutex keeps
// each call's launches together: every kda_scan sits behind the earlier ones on one stream, every
// kda_intra behind the earlier ones on the other, in the same order, so the kda_intra a kda_scan
// waits for only has kernels in front of it that wait for nothing.
struct CallerStream {                       // what is known about one caller's stream handle
    hipStream_t handle = nullptr;
    int state = 0;                          // 0 free, 1 asked, 2 runs beside the kda_intra stream, 3 does not
    uint32_t token = 0;
    hipEvent_t answered = nullptr;
};

struct OverlapGate {
    std::mutex mu;                          // guards everything below
    SideStream side;
    CallerStream callers[kCallerSlots];
    uint32_t *answers = nullptr;            // pinned host memory, one word per slot
    uint32_t *probe_words = nullptr;        // device address of g_caller_probe
    uint32_t next_token = 1;
    bool tried = false, ok = false;
    // the last overlapped call: which caller's stream it came down (side.join tells when its kda_intra is over)
    hipStream_t last_stream = nullptr;
    bool last_recorded = false;
};

// Called with the mutex held.  May the caller's stream itself carry kda_scan (no hop through a helper
// stream in front of it)?  Only once a probe has shown that it runs beside the kda_intra stream;
// the first calls on a stream answer no and start the probe.
static bool caller_runs_beside_intra(OverlapGate *g, hipStream_t stream)
{
    if (!g->tried) {
        g->tried = true;
        void *dev_words = nullptr;
        g->ok = hipHostMalloc(reinterpret_cast<void **>(&g->answers), kCallerSlots * sizeof(uint32_t), hipHostMallocDefault) == hipSuccess &&
                hipGetSymbolAddress(&dev_words, HIP_SYMBOL(g_caller_probe)) == hipSuccess;
        g->probe_words = static_cast<uint32_t *>(dev_words);
        (void)hipGetLastError();
    }
    if (!g->ok) return false;
    CallerStream *free_slot = nullptr;
    for (CallerStream &c : g->callers) {
        if (c.state == 0) { if (!free_slot) free_slot = &c; continue; }
        if (c.handle != stream) continue;
        if (c.state == 1 && hipEventQuery(c.answered) == hipSuccess)
            c.state = (g->answers[&c - g->callers] == c.token) ? 2 : 3;
        (void)hipGetLastError();
        return c.state == 2;
    }
    if (!free_slot) return false;                            // table full: such streams keep the helper pair
    CallerStream &c = *free_slot;
    const int slot = (int)(&c - g->callers);
    if (!c.answered && hipEventCreateWithFlags(&c.answered, hipEventDisableTiming) != hipSuccess) {
        c.answered = nullptr; (void)hipGetLastError(); return false;
    }
    c.handle = stream;
    c.token = g->next_token++;
    hipLaunchKernelGGL(kda_caller_poll_kernel, dim3(1), dim3(1), 0, stream, slot, c.token);
    hipLaunchKernelGGL(kda_caller_set_kernel, dim3(1), dim3(1), 0, g->side.stream, slot, c.token);
    const bool queued = hipMemcpyAsync(&g->answers[slot], g->probe_words + 2 * slot + 1, sizeof(uint32_t),
                                       hipMemcpyDeviceToHost, stream) == hipSuccess &&
                        hipEventRecord(c.answered, stream) == hipSuccess;
    c.state = queued ? 1 : 3;
    (void)hipGetLastError();
    return false;
}

static OverlapGate *overlap_gate()
{
    constexpr int kMaxDevices = 64;
    static OverlapGate table[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return &table[dev];
}

// Called with the gate's mutex held.  The first call on a device synchronises with the helper
// streams (the probe above): not under stream capture, where the overlapped mode is off anyway.
static SideStream *side_stream(OverlapGate *gate)
{
    SideStream *s = &gate->side;
    if (!s->tried) {
        s->tried = true;
        bool ok = hipStreamCreateWithFlags(&s->scan_stream, hipStreamNonBlocking) == hipSuccess &&
                  hipEventCreateWithFlags(&s->fork, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&s->fork_intra, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&s->join, hipEventDisableTiming) == hipSuccess &&
                  hipEventCreateWithFlags(&s->join_scan, hipEventDisableTiming) == hipSuccess;
        // candidates that share the scan stream's queue are kept alive, so that the runtime hands
        // the next one another queue
        for (int attempt = 0; ok && attempt < 8 && !s->stream; ++attempt) {
            hipStream_t cand = nullptr;
            if (hipStreamCreateWithFlags(&cand, hipStreamNonBlocking) != hipSuccess) break;
            if (streams_run_together(s->scan_stream, cand)) s->stream = cand;
        }
        s->ok = ok && s->stream != nullptr;
        (void)hipGetLastError();
    }
    return s->ok ? s : nullptr;
}

}  // namespace mfma

size_t chunk_mfma_workspace_size(const kda_dims *d, bool minimal, bool gate)
{
    if (d->num_seqs == 0 || d->heads == 0 || d->seqlen == 0) return 0;
    if (minimal) {
        // four chunk indices per segment keep the launches from being pure overhead
        const int64_t maxc = mfma::max_chunks_per_seq(d);
        return mfma::plan_with(d, maxc < 4 ? maxc : 4, gate).total_bytes;
    }
    return mfma::make_plan(d, 0, true, gate).total_bytes;
}

size_t chunk_mfma_status_offset(const kda_dims *d, size_t workspace_bytes)
{
    return mfma::make_plan(d, workspace_bytes, false, false).status_offset;
}

kda_status chunk_mfma_dispatch(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                               const void *q, const void *k,
                               const void *v, const void *log_alpha, const void *beta, const float *h0,
                               const int32_t *cu, void *o, float *hT, void *workspace,
                               size_t workspace_bytes, bool scalar_gate, hipStream_t stream)
{
    using namespace mfma;
    // kda_intra for (slots handed over to a running kda_scan, raw inputs, one decay per head)
    auto pick_intra = [&](bool handoff) {
        if (scalar_gate) return handoff ? kda_intra_kernel<true, false, true> : kda_intra_kernel<false, false, true>;
        if (pro) return handoff ? kda_intra_kernel<true, true> : kda_intra_kernel<false, true>;
        return handoff ? kda_intra_kernel<true, false> : kda_intra_kernel<false, false>;
    };
    RawParams raw = {nullptr, nullptr, 0.f};
    if (pro) { raw.a_scale = pro->a_scale; raw.dt_bias = pro->dt_bias; raw.eps = pro->l2norm_eps; }
    const int out_bf16 = d->out_dtype == KDA_BF16;
    EpiParams ep = {nullptr, nullptr, 0.f, out_bf16, nullptr};
    if (epi) { ep.gate = static_cast<const uint16_t *>(epi->gate); ep.norm_w = epi->norm_weight; ep.eps = epi->rms_eps; }
    if (d->seqlen == 0) {
        // nothing to scan: the final state is the initial one
        if (hT && hT != h0) {
            const size_t bytes = (size_t)d->num_seqs * d->heads * D * D * sizeof(float);
            hipError_t e = hipSuccess;
            if (h0) {
                e = hipMemcpyAsync(hT, h0, bytes, hipMemcpyDeviceToDevice, stream);
            } else {
                // (a fill kernel rather than a memset: the call may be captured into a graph)
                const int64_t words = (int64_t)(bytes / 4);
                uint32_t *dst = reinterpret_cast<uint32_t *>(hT);
                hipLaunchKernelGGL(kda_fill_u32_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, dst,
                                   words, 0u, dst);
                e = hipGetLastError();
            }
            if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "state copy: %s", hipGetErrorString(e));
        }
        return KDA_OK;
    }
    const SegPlan plan = make_plan(d, workspace_bytes, false, epi != nullptr);
    if (plan.total_bytes > workspace_bytes)
        return fail(KDA_ERR_WORKSPACE, "workspace has %zu bytes, segment plan needs %zu", workspace_bytes,
                    plan.total_bytes);
    if (d->num_seqs > 65535)
        return fail(KDA_ERR_UNSUPPORTED, "more than 65535 sequences in one call: %d", d->num_seqs);
    if ((int64_t)d->num_seqs * d->heads > 0x7fffffffLL)
        return fail(KDA_ERR_UNSUPPORTED, "num_seqs * heads exceeds 2^31 - 1");

    const size_t scan_lds = (size_t)scan::kLds;
    if (!reserve_lds())
        return fail(KDA_ERR_LAUNCH, "cannot reserve LDS for the prefill kernels (%d, %d bytes)", kIntraLds,
                    (int)scan_lds);

    uint8_t *base = static_cast<uint8_t *>(workspace);
    uint8_t *ws = base + plan.slots_offset;
    float *carry = hT ? hT : reinterpret_cast<float *>(base + plan.carry_offset);
    uint32_t *flags = reinterpret_cast<uint32_t *>(base + plan.flags_offset);
    uint32_t *status = reinterpret_cast<uint32_t *>(base + plan.status_offset);
    uint8_t *gate_ws = epi ? base + plan.gate_offset : nullptr;
    ep.gate_ws = gate_ws;
    const uint16_t *q16 = static_cast<const uint16_t *>(q), *k16 = static_cast<const uint16_t *>(k),
                   *v16 = static_cast<const uint16_t *>(v), *g16 = static_cast<const uint16_t *>(log_alpha),
                   *b16 = static_cast<const uint16_t *>(beta);
    const unsigned streams = (unsigned)((int64_t)d->num_seqs * d->heads);
    const dim3 intra_grid_serial((unsigned)d->heads, (unsigned)plan.seg_chunks, (unsigned)d->num_seqs);
    const dim3 intra_grid_overlap((unsigned)d->heads, (unsigned)d->num_seqs, (unsigned)plan.seg_chunks);

    // Overlapped mode: kda_intra runs on a helper stream while kda_scan, on the caller's stream,
    // consumes each slot as soon as its flag is up.  kda_scan keeps one compute unit per
    // (sequence, head) busy for the whole call, and kda_intra, the larger half of the work, has
    // to live on the rest (it never waits for anything, which is what rules out a deadlock):
    // measured on 64 to 192 pairs, running side by side wins up to a third of the compute units
    // (80 pairs of 256: 0.38 against 0.40 ms) and loses beyond (96: 0.45 against 0.44 ms; 192:
    // 1.54 against 0.69 ms), where the kernels run one after the other.
    // Not while the caller's stream is being captured into a graph: a captured kda_scan could be
    // replayed by a runtime that does not start the other branch at the same time.
    SideStream *side = nullptr;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) { capture = hipStreamCaptureStatusNone; (void)hipGetLastError(); }
    const int cus = compute_units();
    if (cus <= 0) return fail(KDA_ERR_LAUNCH, "cannot query the device");
    OverlapGate *gate = nullptr;
    std::unique_lock<std::mutex> gate_lock;
    bool direct = false;
    if (g_phase_mask == 3 && g_overlap && capture == hipStreamCaptureStatusNone &&
        (int64_t)streams * 3 <= (int64_t)cus && (gate = overlap_gate()) != nullptr) {
        gate_lock = std::unique_lock<std::mutex>(gate->mu);              // held until this call is queued
        side = side_stream(gate);
        // One overlapped call at a time unless they come down the same caller's stream: each keeps a
        // compute unit per (sequence, head) waiting, and several of them together could leave their
        // producers none.
        // (the last one counts as over once its kda_intra is: its kda_scan then waits for nothing more)
        if (side && gate->last_recorded && gate->last_stream != stream) {
            if (hipEventQuery(side->join) != hipSuccess) side = nullptr;
            (void)hipGetLastError();
        }
        if (side) direct = caller_runs_beside_intra(gate, stream);
        if (!side) gate_lock.unlock();
    }
    // kda_scan's stream: the caller's own if it is known to run beside the kda_intra stream (and
    // when nothing overlaps), else the library's
    hipStream_t scan_stream = (side && !direct) ? side->scan_stream : stream;
    auto close_gate = [&]() {                // remember whose overlapped call is in flight
        if (!side) return;
        gate->last_recorded = true;
        gate->last_stream = stream;
    };
    // Both helper streams behind everything queued on the caller's stream -- kda_intra's through
    // kda_scan's: its release then reaches it a little after kda_scan has been handed to the device,
    // so kda_scan's workgroups, which need a whole compute unit each, are placed first (if the 4 096
    // half-unit workgroups of kda_intra fill the device first, kda_scan starts when they are nearly through).
    auto fork = [&]() {
        if (direct)                              // kda_scan follows on the caller's stream itself
            return hipEventRecord(side->fork, stream) == hipSuccess &&
                   hipStreamWaitEvent(side->stream, side->fork, 0) == hipSuccess;
        return hipEventRecord(side->fork, stream) == hipSuccess &&
               hipStreamWaitEvent(side->scan_stream, side->fork, 0) == hipSuccess &&
               hipEventRecord(side->fork_intra, side->scan_stream) == hipSuccess &&
               hipStreamWaitEvent(side->stream, side->fork_intra, 0) == hipSuccess;
    };
    auto join = [&]() {                      // the caller's stream behind the helper streams
        if (direct)
            return hipEventRecord(side->join, side->stream) == hipSuccess &&
                   hipStreamWaitEvent(stream, side->join, 0) == hipSuccess;
        return hipEventRecord(side->join, side->stream) == hipSuccess &&
               hipEventRecord(side->join_scan, side->scan_stream) == hipSuccess &&
               hipStreamWaitEvent(stream, side->join, 0) == hipSuccess &&
               hipStreamWaitEvent(stream, side->join_scan, 0) == hipSuccess;
    };
    double first_ratio = 1.0;
    const int parts = (g_phase_mask == 3 && g_split) ? split_parts(plan, d, cus, g_split, &first_ratio) : 1;

    if (side || parts > 1) {
        // the slot flags (overlapped mode), the counters of the time-split scan (they follow the
        // flags), the status word
        uint8_t *first = base + (side ? plan.flags_offset : plan.split_offset);
        const uint8_t *end = base + (parts > 1 ? plan.split_offset + kSplitFlagBytes : plan.split_offset);
        const int64_t nfill = (int64_t)(end - first) / 4;
        hipLaunchKernelGGL(kda_fill_u32_kernel, dim3((unsigned)((nfill + 255) / 256 + 1)), dim3(256), 0, stream,
                           reinterpret_cast<uint32_t *>(first), nfill, 0u, status);
    }
    if (parts > 1) {
        // Time-split scan: one launch per time segment, kda_intra beside it in the overlapped mode.
        // ranges: the first one shorter by the ratio of the step times (full scan : passes without output)
        const double ratio = (g_split_ratio > 0.0) ? g_split_ratio : first_ratio;
        int64_t part0_len = (int64_t)((double)plan.seg_chunks * ratio / ((double)(parts - 1) + ratio) + 0.5);
        if (part0_len < 1) part0_len = 1;
        const int64_t part_len = (plan.seg_chunks - part0_len + parts - 2) / (parts - 1);
        const size_t pair_states = (size_t)streams * D * D;
        uint32_t *split_flags = reinterpret_cast<uint32_t *>(base + plan.split_offset);
        float *E = reinterpret_cast<float *>(base + plan.split_offset + kSplitFlagBytes);
        float *Tm = E + kSplitMaxParts * pair_states, *Bm = Tm + kSplitMaxParts * pair_states;
        auto intra = pick_intra(side != nullptr);
        auto split_k = side ? (epi ? kda_scan_split_kernel<true, true> : kda_scan_split_kernel<true, false>)
                            : (epi ? kda_scan_split_kernel<false, true> : kda_scan_split_kernel<false, false>);
        const dim3 intra_grid_split((unsigned)d->heads, (unsigned)d->num_seqs, (unsigned)(parts * part_len));   // z: see kda_intra
        for (int64_t seg = 0; seg < plan.num_segments; ++seg) {
            const float *sin = (seg == 0) ? h0 : carry;
            float *sout = (plan.num_segments > 1 || hT) ? carry : nullptr;
            const uint32_t epoch = (uint32_t)(seg + 1);
            if (seg > 0)    // the counters of the ranges start every segment at zero (the extra word: one of them)
                hipLaunchKernelGGL(kda_fill_u32_kernel, dim3((unsigned)(kSplitFlagBytes / 4 / 256)), dim3(256), 0, stream,
                                   split_flags, (int64_t)(kSplitFlagBytes / 4), 0u, split_flags);
            if (side) {
                if (!fork())
                    return fail(KDA_ERR_LAUNCH, "cannot order the helper streams: %s", hipGetErrorString(hipGetLastError()));
            } else {
                hipLaunchKernelGGL(intra, intra_grid_serial, dim3(256), kIntraLds, stream, q16, k16, v16, g16, b16, cu, ws,
                                   (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg, d->scale,
                                   (uint32_t *)nullptr, 0u, raw, 1, 0, 0, ep.gate, gate_ws);
            }
            hipLaunchKernelGGL(split_k, dim3(streams, (unsigned)(2 * parts - 3)), dim3(512), scan_lds, scan_stream, ws, sin, E,
                               Tm, Bm, sout, cu, o, (int64_t)d->seqlen, (int)d->heads,
                               plan.seg_chunks, seg, part_len, part0_len, parts, flags, epoch, status, split_flags, ep);
            if (side) {
                hipLaunchKernelGGL(intra, intra_grid_split, dim3(256), kIntraLds, side->stream, q16, k16, v16, g16, b16, cu, ws,
                                   (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg, d->scale, flags, epoch, raw,
                                   parts, (int)part_len, (int)part0_len, ep.gate, gate_ws);
                if (!join())
                    return fail(KDA_ERR_LAUNCH, "cannot join the helper streams: %s", hipGetErrorString(hipGetLastError()));
            }
        }
        close_gate();
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "prefill kernels: %s", hipGetErrorString(e));
        return KDA_OK;
    }
    for (int64_t seg = 0; seg < plan.num_segments; ++seg) {
        const float *sin = (seg == 0) ? h0 : carry;
        float *sout = (plan.num_segments > 1 || hT) ? carry : nullptr;
        if (side) {
            // kda_intra of this segment may start once everything queued so far on the caller's
            // stream (the inputs' producers, the flag reset, the previous segment's scan) is done
            const uint32_t epoch = (uint32_t)(seg + 1);
            if (!fork())
                return fail(KDA_ERR_LAUNCH, "cannot order the helper streams: %s", hipGetErrorString(hipGetLastError()));
            auto scan_k = epi ? kda_scan_kernel<true, true> : kda_scan_kernel<true, false>;
            hipLaunchKernelGGL(scan_k, dim3(streams), dim3(512), scan_lds, scan_stream, ws, sin, sout, cu,
                               o, (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg,
                               flags, epoch, status, ep);
            auto intra = pick_intra(true);
            hipLaunchKernelGGL(intra, intra_grid_overlap,
                               dim3(256), kIntraLds, side->stream, q16, k16, v16, g16, b16, cu, ws,
                               (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg, d->scale, flags, epoch, raw, 1, 0, 0, ep.gate, gate_ws);
            if (!join())
                return fail(KDA_ERR_LAUNCH, "cannot join the helper streams: %s", hipGetErrorString(hipGetLastError()));
        } else {
            auto intra = pick_intra(false);
            if (g_phase_mask & 1)
                hipLaunchKernelGGL(intra, intra_grid_serial, dim3(256), kIntraLds, stream, q16, k16, v16, g16, b16, cu, ws,
                                   (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg, d->scale,
                                   (uint32_t *)nullptr, 0u, raw, 1, 0, 0, ep.gate, gate_ws);
            auto scan_k = epi ? kda_scan_kernel<false, true> : kda_scan_kernel<false, false>;
            if (g_phase_mask & 2)
                hipLaunchKernelGGL(scan_k, dim3(streams), dim3(512), scan_lds, stream, ws, sin, sout, cu,
                                   o, (int64_t)d->seqlen, (int)d->heads, plan.seg_chunks, seg,
                                   (const uint32_t *)nullptr, 0u, status, ep);
        }
    }
    close_gate();
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "prefill kernels: %s", hipGetErrorString(e));
    return KDA_OK;
}

}  // namespace kda
