// kda_scan8: the sequential stage of the matrix-core prefill as a workgroup of EIGHT waves on a whole
// compute unit, kept for calls with the fused output gate of Section 4 (the four-wave scan of
// kda_scan4.h, which every other call uses, has no LDS to spare for the gate's reduction).
//
// One workgroup walks the chunks of one (sequence, head).  Wave (c, p) owns the 32-column slice c of
// the state for the two d_k tiles 2p, 2p+1, and the token tile p of V_new and O.  A chunk costs each
// wave 26-28 MFMAs (32x32x16), at the price of two exchanges through LDS per chunk: the fp16 copies
// of S (every wave needs all four d_k tiles as an operand) and of V_new (both token tiles).  All
// other operands stream from the LDS copy of the workspace slot.  The slot of chunk c + 2 is fetched
// into registers while chunk c computes and written to the other LDS stage at the end of chunk
// c + 1, so a fetch has two full steps to arrive.  O is accumulated transposed (operands swapped), so
// a lane owns four consecutive output columns and stores 16 bytes at a time.
#pragma once
#include <type_traits>

#include "kda_scan4.h"

namespace kda {
namespace mfma {

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

// (kFlags and kRole are compiled for false / kRoleFull only: the calls that hand slots over while both stages
// run, and the time-split ranges, belong to the four-wave scan)
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

}  // namespace mfma
}  // namespace kda
