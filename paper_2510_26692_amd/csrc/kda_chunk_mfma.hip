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
#include "kda_intra.h"
#include "kda_prefill_fused.h"

namespace kda {

extern int g_phase_mask;   // diagnostics switches owned by kda_api.hip
extern int g_overlap;
extern int g_split;
extern double g_split_ratio;
extern int g_fused;            // 1: the one-kernel prefill (kda_prefill_fused.hip) wherever it applies
extern int g_producers;        // diagnostic: 0 switches the per-chunk role of the one-kernel prefill off
extern uint64_t g_wait_limit;  // ticks of the 100 MHz wall clock a scan workgroup waits for one slot

namespace mfma {

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
    kda_intra_chunk<kHandoff, kRaw, kScalar>(lds, q, k, v, log_alpha, beta, cu_seqlens, ws, T, H, seg_chunks, seg_index,
                                             scale, ready, epoch, raw, out_gate, gate_ws, h, n, cl);
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
        const int64_t gate_stride = (int64_t)kGateSlotBytes;
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
    const uint8_t *slot0 = ws + (((int64_t)n * H + h) * seg_chunks) * (int64_t)kSlotBytes;
    const int64_t slot_stride = (int64_t)kSlotBytes;

    if (kEpi && threadIdx.x < D)     // RMSNorm weights: read by every step after its first barrier
        reinterpret_cast<float *>(lds + scan::kNormW)[threadIdx.x] = epi.norm_w ? epi.norm_w[threadIdx.x] : 1.f;
    const uint32_t *flag0 = kFlags ? ready + (int64_t)blockIdx.x * seg_chunks : nullptr;
    // nothing is waited for without flags: leave a clean status word for kda_chunk_fwd_check
    if (!kFlags && status && blockIdx.x == 0 && threadIdx.x == 0) *status = 0;

    if (kEpi) epi.gate_ws += (((int64_t)n * H + h) * seg_chunks) * (int64_t)kGateSlotBytes;   // this pair's first slot
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
    const int64_t slot_stride = (int64_t)kSlotBytes;
    if (kEpi && threadIdx.x < D)     // RMSNorm weights of the output gate (beyond what the fold uses of the LDS)
        reinterpret_cast<float *>(lds + scan::kNormW)[threadIdx.x] = epi.norm_w ? epi.norm_w[threadIdx.x] : 1.f;
    const uint8_t *gate_base = epi.gate_ws;

    // (the output gate concerns the full scan only; the passes without output ignore it)
#define KDA_SCAN_PART(ROLE, EPI)                                                                                  \
    if (EPI) epi.gate_ws = gate_base + (((int64_t)n * H + h) * seg_chunks + c_begin) * (int64_t)kGateSlotBytes;   \
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
        const uint8_t *slot0 = ws + (((int64_t)n * H + h) * seg_chunks + c_begin) * (int64_t)kSlotBytes;
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
        const uint8_t *slot0 = ws + (((int64_t)n * H + h) * seg_chunks + c_begin) * (int64_t)kSlotBytes;
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

// The same decision for the one-kernel prefill, where every workgroup of either stage takes half a compute
// unit: the scan workgroups of a split launch may take three eighths of those slots.  Estimate
// (microseconds, measured on MI355X): a step of the four-wave scan 2.4, a chunk of the per-chunk stage
// 15.6 on one slot.
static int split_parts_fused(const SegPlan &plan, const kda_dims *d, int cus, int forced, double *first_ratio)
{
    *first_ratio = 1.0;
    int64_t maxc = max_chunks_per_seq(d);
    if (maxc > plan.seg_chunks) maxc = plan.seg_chunks;
    const int64_t pairs = (int64_t)d->num_seqs * d->heads;
    const int64_t slots = 2 * (int64_t)cus;
    if (pairs > kSplitMaxPairs || maxc < kSplitMinChunks || pairs >= slots) return 1;
    const double step = 2.4, item = 15.6;
    const double items = (double)pairs * (double)maxc;
    const double t_scan = (double)maxc * step, t_intra1 = items * item / (double)(slots - pairs);
    double best = t_scan > t_intra1 ? t_scan : t_intra1;
    int parts = 1;
    for (int p = 3; p <= kSplitMaxParts; ++p) {
        const int64_t len = (maxc + p - 1) / p;
        if (pairs * (2 * p - 3) * 8 > slots * 3 || len < 8) continue;
        const double phase = (double)len * step;
        const double t_intra = items * item / (double)(slots - pairs * (2 * p - 3));
        const double fed = t_intra * (double)(p - 1) / (double)p;
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

    // One launch per time segment, both stages as roles of one kernel (kda_prefill_fused.hip).
    if (g_fused && g_phase_mask == 3 && !epi) {
        double fratio = 1.0;
        const int fparts = g_split ? split_parts_fused(plan, d, cus, g_split, &fratio) : 1;
        const double ratio = (g_split_ratio > 0.0) ? g_split_ratio : fratio;
        int64_t part0_len = 0, part_len = 0;
        if (fparts > 1) {
            part0_len = (int64_t)((double)plan.seg_chunks * ratio / ((double)(fparts - 1) + ratio) + 0.5);
            if (part0_len < 1) part0_len = 1;
            part_len = (plan.seg_chunks - part0_len + fparts - 2) / (fparts - 1);
        }
        const size_t pair_states = (size_t)streams * D * D;
        for (int64_t seg = 0; seg < plan.num_segments; ++seg) {
            FusedLaunch L{};
            FusedArgs &a = L.args;
            a.q = q16; a.k = k16; a.v = v16; a.log_alpha = g16; a.beta = b16; a.cu = cu;
            a.state_in = (seg == 0) ? h0 : carry;
            a.state_out = (plan.num_segments > 1 || hT) ? carry : nullptr;
            a.o = o; a.ws = ws; a.ready = flags; a.status = status;
            a.T = d->seqlen; a.pairs = streams; a.seg_chunks = plan.seg_chunks; a.seg_index = seg;
            int64_t left = max_chunks_per_seq(d) - seg * plan.seg_chunks;
            a.launch_chunks = left < plan.seg_chunks ? left : plan.seg_chunks;
            a.wait_limit = g_wait_limit; a.H = d->heads; a.scale = d->scale; a.epoch = (uint32_t)(seg + 1);
            a.producers = g_producers; a.raw = raw;
            a.split.parts = fparts; a.split.part_len = part_len; a.split.part0_len = part0_len;
            a.split.flags = reinterpret_cast<uint32_t *>(base + plan.split_offset);
            a.split.E = reinterpret_cast<float *>(base + plan.split_offset + kSplitFlagBytes);
            a.split.Tm = a.split.E + kSplitMaxParts * pair_states;
            a.split.Bm = a.split.Tm + kSplitMaxParts * pair_states;
            L.raw = pro != nullptr; L.scalar_gate = scalar_gate; L.out_bf16 = out_bf16 != 0;
            L.reset_flags = seg == 0 && !(g_producers == 0 && getenv("KDA_DBG_KEEPFLAGS"));
            // (the counters of the time-split scan follow the slot flags: one fill clears both)
            L.num_flags = fparts > 1 ? (int64_t)((plan.split_offset + kSplitFlagBytes - plan.flags_offset) / 4)
                                     : (int64_t)plan.seg_chunks * streams;
            L.reset_split = fparts > 1 && seg > 0;
            const kda_status st = launch_prefill_fused(L, stream);
            if (st != KDA_OK) return st;
        }
        return KDA_OK;
    }
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
