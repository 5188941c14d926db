// kda_intra: the per-chunk stage of the matrix-core prefill (Section 3.1), as a device function
// that a kernel calls with the (head, sequence, chunk) of its workgroup.  It forms the running
// log-decay G, the two intra-chunk matrices A_kk and A_qk, the UT transform
// M = (I + StrictTril(Diag(beta) A_kk))^-1 Diag(beta) by forward substitution, W = M (Gamma.K),
// U = M V and the decay-scaled operands Gamma.Q and Gamma^{i->C}.K, and leaves them in the chunk's
// workspace slot in MFMA register order (kda_mfma_layout.h).
//
// Matrix-core operands are fp16 (unit roundoff 2^-11), accumulation is fp32.  bf16 inputs convert
// to fp16 exactly while their magnitude lies in [2^-14, 65504] (or is zero); derived operands are rounded.
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
#pragma once
#include "kda_common.h"
#include "kda_mfma_layout.h"

namespace kda {
namespace mfma {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kMaxKeyNorm2 = 16.0f;  // |k_t|^2 up to which the fp16 operands are safe (entries then stay below 4)
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

// Input rows are read through a descriptor that covers exactly the bytes that may be read: the hardware
// returns zeros for an offset beyond it (a padding token of a ragged chunk).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_resource(const void *base, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 rows_load16(__amdgpu_buffer_rsrc_t rs, int off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
}
__device__ __forceinline__ uint16_t rows_load2(__amdgpu_buffer_rsrc_t rs, int off)
{
    return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
}

// A value that is the same in every lane of the wave, moved to scalar registers.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ int64_t uni64(int64_t x)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
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

// What the per-chunk stage reads and writes, the same for every chunk of a launch.
struct IntraArgs {
    const uint16_t *q, *k, *v, *log_alpha, *beta;    // bf16 inputs (log_alpha: [B,T,H,128], or [B,T,H] with kScalar)
    const int32_t *cu_seqlens;                       // NULL: sequences of T tokens
    uint8_t *ws;                                     // slots
    int64_t T;
    int H;
    int64_t seg_chunks, seg_index;                   // time segment: chunk indices seg_index * seg_chunks + [0, seg_chunks)
    float scale;
    uint32_t *ready;                                 // kHandoff: one flag per slot
    uint32_t epoch;                                  //           value of a raised flag
    RawParams raw;
    const uint16_t *out_gate;                        // fused output gate: logits [B,T,H,128] or NULL
    uint8_t *gate_ws;                                //   slots of the gate factors w_j Sigmoid(g_tj), fp16, kGateSlotBytes each
    const float *gate_norm_w;                        //   RMSNorm weights [128] or NULL (= ones)
    uint32_t *status;                                // may be NULL
};
// One chunk of one (sequence, head): cl is the chunk index inside the time segment; cl < 0: nothing to do.
struct IntraItem {
    int h, n;
    int64_t cl;
};

// Workgroup of 256 threads (four waves), kIntraLds bytes of LDS at `lds`.  The workgroup works through the items
// item_at(0), .., item_at(count - 1) one after the other; the inputs of an item are fetched while the item before
// it is still being computed, so only the first fetch of a workgroup is waited for in full.  item_at must
// return the same item in every thread.  Every thread of the workgroup must make the call (barriers inside).
// status: bit 2 is raised when a key of the chunk has |k_t|^2 > kMaxKeyNorm2, beyond which the fp16
// operands may overflow and the UT transform loses accuracy (the paper's keys are L2-normalised, Section 4).
template <bool kHandoff, bool kRaw, bool kScalar, typename ItemAt>
__device__ __forceinline__
void kda_intra_items(uint8_t *lds, const IntraArgs &A, int count, ItemAt item_at)
{
    // (the wave index is the same in all lanes: telling the compiler so turns the per-wave cases
    // below into scalar branches instead of masked vector code)
    constexpr int kPolicy = kHandoff ? kCacheDevice : 0;
    const uint16_t *__restrict__ q = A.q, *__restrict__ k = A.k, *__restrict__ v = A.v;
    const uint16_t *__restrict__ log_alpha = A.log_alpha, *__restrict__ beta = A.beta, *__restrict__ out_gate = A.out_gate;
    uint8_t *__restrict__ ws = A.ws, *__restrict__ gate_ws = A.gate_ws;
    const int H = A.H;
    const int64_t seg_chunks = A.seg_chunks;
    const float scale = A.scale;
    const RawParams raw = A.raw;
    uint32_t *status = A.status;
    const int row_pitch = H * D * 2;                          // bytes between consecutive tokens of an input

    // Where an item's data is: slots are laid out pair by pair, a pair's chunks one after the other (the
    // sequential stage then walks one contiguous range of memory per (sequence, head)).  row0: this head's row
    // of the chunk's first token in the [token][head][128] inputs; row_bytes: from there to the end of the
    // last valid token's row; head_bytes: the same for the [token][head] inputs.  An item that does not exist
    // (no such chunk in the segment or the sequence) has valid = false and row_bytes = head_bytes = 0.
    struct Loc {
        bool valid;
        int h, nv, row_bytes, head_bytes;
        int64_t slot, tok0, row0;
    };
    auto locate = [&](const IntraItem it) __attribute__((always_inline)) {
        Loc L;
        L.valid = false; L.h = it.h; L.nv = 0; L.row_bytes = 0; L.head_bytes = 0;
        L.slot = 0; L.tok0 = 0; L.row0 = 0;
        if (it.cl >= 0 && it.cl < seg_chunks) {
            const int64_t ci = A.seg_index * seg_chunks + it.cl;
            int64_t tok_base, len;
            if (A.cu_seqlens) { tok_base = A.cu_seqlens[it.n]; len = (int64_t)A.cu_seqlens[it.n + 1] - tok_base; }
            else              { tok_base = (int64_t)it.n * A.T; len = A.T; }
            if (ci * kChunk < len) {
                L.valid = true;
                L.nv = (int)((len - ci * kChunk < kChunk) ? (len - ci * kChunk) : kChunk);
                L.slot = ((int64_t)it.n * H + it.h) * seg_chunks + it.cl;
                L.tok0 = tok_base + ci * kChunk;
                L.row0 = (L.tok0 * H + it.h) * (int64_t)D;
                L.row_bytes = (L.nv - 1) * row_pitch + D * 2;
                L.head_bytes = ((L.nv - 1) * H + 1) * 2;
            }
        }
        // (the same in every lane: kept in scalar registers)
        L.h = uni(L.h); L.nv = uni(L.nv); L.row_bytes = uni(L.row_bytes); L.head_bytes = uni(L.head_bytes);
        L.slot = uni64(L.slot); L.tok0 = uni64(L.tok0); L.row0 = uni64(L.row0);
        L.valid = uni((int)L.valid) != 0;
        return L;
    };
    // The inputs the first phases need, 16 bytes (8 channels) per ks and tensor, all through descriptors that
    // end with the chunk's last valid token: a token beyond it (and every token of an item that does not
    // exist) reads as zeros, with no branch around a load and nothing for a load to wait for.
    // (log_alpha first: the running sum waits for it, k and q are needed later)
    u32x4 kraw[4], qraw[4], graw[4];
    uint32_t beta_raw = 0, gscalar_raw = 0;                  // beta of token tid % 64; kScalar: log alpha of this lane's token
    auto fetch = [&](const Loc &L, const int tid) __attribute__((always_inline)) {
        const int tok = (tid & 63 & 15) + 16 * (tid >> 6), g = (tid & 63) >> 4;
        const int off = tok * row_pitch + 16 * g;
        const __amdgpu_buffer_rsrc_t rg = rows_resource(log_alpha + L.row0, kScalar ? 0 : L.row_bytes);
        const __amdgpu_buffer_rsrc_t rk = rows_resource(k + L.row0, L.row_bytes), rq = rows_resource(q + L.row0, L.row_bytes);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) graw[ks] = rows_load16(rg, off + 64 * ks);
        if (kScalar) gscalar_raw = rows_load2(rows_resource(log_alpha + (L.tok0 * H + L.h), L.head_bytes), tok * H * 2);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kraw[ks] = rows_load16(rk, off + 64 * ks);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qraw[ks] = rows_load16(rq, off + 64 * ks);
        beta_raw = rows_load2(rows_resource(beta + (L.tok0 * H + L.h), L.head_bytes), (tid & 63) * H * 2);
    };

    // Each item is computed in two halves, and the loop is rotated by one half: a pass fetches the inputs of
    // its item, finishes the item before it (which does not touch them) and then computes the first half of
    // its own, so a fetch has the second half of an item, a third of the whole, to arrive, and no register
    // holds fetched data from one pass of the loop to the next.  Between its halves an item lives in LDS and
    // in the A_kk and A_qk tiles (R, I), I = 0..R, of this wave.
    f32x4 res_kk[4], res_qk[4];
    Loc prev = locate(IntraItem{0, 0, -1}), cur = locate(item_at(0));
    for (int item = 0; item <= count; ++item) {
        // (the thread index is made opaque once per pass: what is derived from it, addresses above all, is then
        // computed where it is used instead of being carried in registers across the whole loop)
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
        const int R = wave, m = lane & 15, g = lane >> 4;
        const int tok = 16 * R + m;
        fetch(cur, tid);                                         // (nothing is read for an item that does not exist)
        float *sTot = reinterpret_cast<float *>(lds + kTot);
        float *sBeta = reinterpret_cast<float *>(lds + kBeta);
        uint32_t *sStrong = reinterpret_cast<uint32_t *>(lds + kStrong);
        float *sTab = reinterpret_cast<float *>(lds + kTab);     // [7][4][128]: P, E, Tinv, iA, iB, shifted total, row shift


        if (prev.valid) {                                        // ---- second half of the item before ----
            const int h = prev.h, nv = prev.nv, row_bytes = prev.row_bytes;
            const int64_t slot = prev.slot, row0 = prev.row0;
            const __amdgpu_buffer_rsrc_t out = slot_resource(ws + slot * (int64_t)kSlotBytes);
            (void)h;
            // ---- output gate (fused epilogue): the chunk's gate factors go out in the accumulator order of the
            // sequential stage, which reads them like any other part of the slot.  Done first thing in the second half
            // of the chunk, where few registers are in use, and fenced off from the scheduler so that it stays there.
            if (out_gate) {
                __builtin_amdgcn_sched_barrier(0);
                u32x4 ograw[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
                    ograw[i] = rows_load16(rows_resource(out_gate + row0, row_bytes), tokv * row_pitch + 16 * cg);
                }
                // piece (token, 8 columns 8 cg ..) = column group q = cg % 4 of tile (token / 32, cg / 4): its
                // first four columns belong to lane (token % 32, hh = 0), the other four to lane (.., hh = 1)
                const __amdgpu_buffer_rsrc_t gout = __builtin_amdgcn_make_buffer_rsrc(
                    gate_ws + slot * (int64_t)kGateSlotBytes, 0, kGateSlotBytes, 0x00020000);
                float gate_w[8];                                     // RMSNorm weights of this thread's 8 columns (the same in all four pieces)
#pragma unroll
                for (int e = 0; e < 8; ++e) gate_w[e] = A.gate_norm_w ? A.gate_norm_w[8 * (tid & 15) + e] : 1.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int u = tid + 256 * i, tokv = u >> 4, cg = u & 15;
                    const int base = ((tokv >> 5) * 4 + (cg >> 2)) * kGateTileBytes + ((cg & 3) >> 1) * 1024 + (tokv & 31) * 16 +
                                     (cg & 1) * 8;
                    // what leaves is the factor the gate multiplies the normalised o by, w_j Sigmoid(g_tj), as fp16 (it lies
                    // in (0, |w_j|); the 2^-11 of its rounding is a quarter of the tolerance and comes off the sequential
                    // stage's critical path, which would otherwise evaluate 32 exponentials per lane and chunk)
                    uint32_t f[4];
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        float g0, g1;
                        unpack_bf16x2(ograw[i][w], g0, g1);
                        f[w] = pack_h2(gate_w[2 * w] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-g0 * kLog2e)),
                                       gate_w[2 * w + 1] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-g1 * kLog2e)));
                    }
                    const u32x2 lo = {f[0], f[1]}, hi = {f[2], f[3]};
                    slot_store8<kPolicy>(gout, base, lo);
                    slot_store8<kPolicy>(gout, base + 32 * 16, hi);
                }
                __builtin_amdgcn_sched_barrier(0);
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
                vraw[i] = rows_load16(rows_resource(v + row0, row_bytes), tokv * row_pitch + 16 * cg);
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
                    __hip_atomic_store(A.ready + slot, A.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (cur.valid) {
                __syncthreads();                                     // the tiles in LDS are free for the next item
            }
        }

        if (cur.valid) {                                         // ---- first half of this pass's item ----
            const int h = cur.h, nv = cur.nv, row_bytes = cur.row_bytes;
            const int64_t slot = cur.slot, row0 = cur.row0;
            const __amdgpu_buffer_rsrc_t out = slot_resource(ws + slot * (int64_t)kSlotBytes);
            // ---- this item's inputs were fetched while the item before it was computed ----
            const float gscalar = bf16_bits_to_float((uint16_t)gscalar_raw);    // kScalar: log alpha of this lane's token
            const float beta_tok = bf16_bits_to_float((uint16_t)beta_raw);      // beta of token tid (threads 0..63)
            static_assert(!(kRaw && kScalar), "the fused prologue is built for the per-channel gate");
            if (tid < kChunk) {
                float b = beta_tok;
                if (kRaw) b = (tid < nv) ? __builtin_amdgcn_rcpf(1.f + fast_exp2(-b * kLog2e)) : 0.f;   // Sigmoid
                sBeta[tid] = b;
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
                    // the diagonal of the diagonal tile is |k_t|^2: the domain check of the keys costs a few compares
                    if (status) {
                        bool bad = false;
#pragma unroll
                        for (int j = 0; j < 4; ++j) bad |= (4 * g + j == m) && !(akk[j] <= kMaxKeyNorm2);
                        if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0)
                            __hip_atomic_fetch_or(status, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    // (written through constant indices: an array indexed by the wave number would be placed in scratch memory)
#pragma unroll
                    for (int I = 0; I < 4; ++I)
                        if (I == R) { res_kk[I] = akk; res_qk[I] = aqk; }
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
                            // (the running sum of the slot's channel is formed again from the input: holding all 32 sums up to here
                            // for the sake of this rare path would keep them in registers across the operand loop, the tightest
                            // point of the kernel; only differences of it are used, so the row shift is not needed)
                            float Ge = bf16_bits_to_float(rows_load2(rows_resource(log_alpha + row0, row_bytes),
                                                                     tok * row_pitch + 16 * g + 64 * ks + 2 * e));
                            if (kRaw) {
                                const float be = raw.dt_bias ? raw.dt_bias[h * D + 32 * ks + 8 * g + e] : 0.f;
                                Ge = (tok < nv) ? log2_alpha_from_gate(Ge + be, a_scale) : 0.f;
                            } else {
                                Ge *= kLog2e;
                            }
                            Ge += row_shr<1>(Ge); Ge += row_shr<2>(Ge); Ge += row_shr<4>(Ge); Ge += row_shr<8>(Ge);
                            // (k and q of the slot are read again: keeping the raw inputs in registers up to here for
                            // the sake of this rare path would cost the common one 24 registers at its tightest point)
                            const int woff = tok * row_pitch + 16 * g + 64 * ks + 4 * (e >> 1);
                            const uint32_t kw = __builtin_amdgcn_raw_buffer_load_b32(rows_resource(k + row0, row_bytes), woff, 0, 0);
                            const uint32_t qw = __builtin_amdgcn_raw_buffer_load_b32(rows_resource(q + row0, row_bytes), woff, 0, 0);
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
                // the diagonal of the diagonal tile is |k_t|^2: the domain check of the keys costs a few compares
                if (status) {
                    bool bad = false;
#pragma unroll
                    for (int j = 0; j < 4; ++j) bad |= (4 * g + j == m) && !(akk[j] <= kMaxKeyNorm2);
                    if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0)
                        __hip_atomic_fetch_or(status, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                // (written through constant indices: an array indexed by the wave number would be placed in scratch memory)
#pragma unroll
                    for (int I = 0; I < 4; ++I)
                        if (I == R) { res_kk[I] = akk; res_qk[I] = aqk; }
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

        }
        prev = cur;
        cur = (item + 1 < count) ? locate(item_at(item + 1)) : locate(IntraItem{0, 0, -1});
    }
}

}  // namespace mfma
}  // namespace kda
