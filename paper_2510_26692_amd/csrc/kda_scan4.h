// kda_scan4: the sequential stage of the matrix-core prefill (Section 3.1: chunk state update,
// inter- and intra-chunk output), as a device function for a workgroup of FOUR waves that needs half
// a compute unit (80 KiB of LDS, at most 256 registers per lane), so that it shares a compute unit
// with a workgroup of the per-chunk stage or with another one of its kind.
//
// Per chunk of one (sequence, head), with the operands the per-chunk stage left in the slot:
//
//     V_new = U - W S          O = (Gamma.Q) S + Tril(A_qk) V_new
//     S <- Diag(gamma^C) S + (Gamma^{i->C}.K)^T V_new
//
// Every column of S is an independent recurrence.  Wave c owns the 32 columns 32 c .. 32 c + 31 of
// S for ALL of d_k (four 32x32 accumulator tiles), and with them the same columns of V_new and O
// for both 32-token tiles: nothing is exchanged between the waves, and the B operands of every
// product (S, V_new as fp16) come straight out of the wave's own accumulators.  What the waves
// share is read-only: the A operands W, Gamma.Q, (Gamma^{i->C}.K)^T and Tril(A_qk), 54 fragments of
// 1 KiB per chunk, which all four waves read from LDS.
//
// Operand path.  The slot is cut into four pieces in the order a step consumes them: W (16 KiB),
// Gamma.Q (16 KiB), K^T (16 KiB) and a small one (A_qk and gamma^C, 8 KiB).  LDS holds a ring of
// four 16 KiB regions and two small ones.  Pieces arrive by LDS-direct loads (global_load_lds:
// no registers in between); a region is refilled as soon as all waves are through with it, with
// the piece that is consumed one whole step later, so about 54 KiB are in flight at any time.  A
// step has three phases (V_new; O; state update) and one workgroup barrier in front of each, which
// says two things at once: every wave's part of the phase's piece has landed, and every wave is done
// reading the piece of the phase before.  The wave's own U tile (4 KiB) travels through registers.
//
// All vector-memory instructions of the loop are issued from inline assembly in a fixed order
// and waited for with explicit vmcnt counts (they retire in issue order), because a wait that the
// compiler derives cannot tell the loads apart and would drain the whole prefetch queue at every
// use.  The registers that such a load writes are defined and consumed inside one loop iteration.
#pragma once
#include <type_traits>

#include "kda_intra.h"

namespace kda {
namespace mfma {

// What one pass over a range of chunks computes (the time-split scan uses the last two):
//   kRoleFull   the scan itself: state from state_in (zero if NULL), outputs written
//   kRoleT      the d_k x d_k transition of the range: starts from the identity, drops U (the
//               recurrence is affine in the state: S_out = T S_in + B), writes no output
//   kRoleB      the offset of the range: starts from zero, keeps U, writes no output
// A kRoleT pass returns whether the transition it ended with is exactly zero (every other pass: false).
constexpr int kRoleFull = 0, kRoleT = 1, kRoleB = 2;

namespace scan4 {


constexpr int kBig = 16 * kFragBytes;                       // W, Gamma.Q or K^T of one chunk
constexpr int kSmall = 8 * kFragBytes;                      // Tril(A_qk), gamma^C (and the first bytes of U, unused)
constexpr int kSmallRegions = 4 * kBig;                     // byte offset of the two small regions
constexpr int kLds = kSmallRegions + 2 * kSmall;            // 81920
// The tail of a small region, behind Tril(A_qk) and gamma^C, receives bytes nobody reads; while its step is being
// worked on it carries the partial mean squares of the output gate: [token tile][wave][32 tokens] fp32.
constexpr int kGateRed = kOffGc - kOffAqk + D * 4;          // 6656
static_assert(kGateRed + 2 * 4 * 32 * 4 <= kSmall, "the partial sums fit the tail of the small region");
static_assert(kOffQp == kBig && kOffKt == 2 * kBig && kOffAqk == 3 * kBig, "pieces follow the slot layout");
static_assert(kOffAqk + kSmall <= kSlotBytes && kOffGc + D * 4 <= kOffAqk + kSmall, "the small piece stays inside the slot");
static_assert(kLds <= 80 * 1024, "two workgroups must fit a compute unit");

// compile-time loop: f(integral_constant<int, I>) for I in [0, N)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// ---- vector memory from inline assembly (device-scope policy sc1: the slots are written by
// workgroups of the same launch, on any die) ----
// Four LDS-direct loads: lane L of the wave moves 16 bytes from src + voff + 1024 j to LDS byte
// m0 + 1024 j + 16 L, j = 0..3 (the instruction offset applies to both addresses).
__device__ __forceinline__ void dma4(uint32_t m0, uint32_t voff, const uint8_t *src)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2 sc1\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:1024 sc1\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:2048 sc1\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:3072 sc1"
                 :: "s"(m0), "v"(voff), "s"(src) : "memory", "m0");
}
__device__ __forceinline__ void dma2(uint32_t m0, uint32_t voff, const uint8_t *src)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2 sc1\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:1024 sc1"
                 :: "s"(m0), "v"(voff), "s"(src) : "memory", "m0");
}
// One LDS-direct load of 16 bytes per lane: LDS byte m0 + 16 L <- src[voff(L)].
__device__ __forceinline__ void dma1(uint32_t m0, uint32_t voff, const uint8_t *src)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2 sc1"
                 :: "s"(m0), "v"(voff), "s"(src) : "memory", "m0");
}
__device__ __forceinline__ void load1(u32x4 &a, uint32_t voff, const uint8_t *src)
{
    asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=&v"(a) : "v"(voff), "s"(src) : "memory");
}
// lane i of each quad of four lanes receives the value of lane kSel[i] of the quad
template <int kCtrl> __device__ __forceinline__ float quad_perm(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xf, 0xf, true));
}
// 4 x 4 transpose across the four lanes of a quad, one component: on entry r[q] belongs to register
// group q of this lane, on exit r[i] is what lane 4 (lane / 4) + i held for group lane % 4.
__device__ __forceinline__ void quad_transpose(float (&r)[4], int lane)
{
    const bool l0 = lane & 1, l1 = lane & 2;
    // 2 x 2 blocks across lanes that differ in bit 0 (quad_perm 1,0,3,2), then across bit 1 (2,3,0,1):
    // each lane sends the register its partner wants and puts what it receives in that register's place
#pragma unroll
    for (int b = 0; b < 4; b += 2) {
        const float t = quad_perm<0xB1>(l0 ? r[b] : r[b + 1]);
        if (l0) r[b] = t; else r[b + 1] = t;
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const float t = quad_perm<0x4E>(l1 ? r[b] : r[b + 2]);
        if (l1) r[b] = t; else r[b + 2] = t;
    }
}
// Two 16-byte loads into registers (valid only after the matching wait).
__device__ __forceinline__ void load2(u32x4 &a, u32x4 &b, uint32_t voff, const uint8_t *src)
{
    asm volatile("global_load_dwordx4 %0, %2, %3 sc1\n\t"
                 "global_load_dwordx4 %1, %2, %3 offset:1024 sc1"
                 : "=&v"(a), "=&v"(b) : "v"(voff), "s"(src) : "memory");
}
__device__ __forceinline__ void load_word(uint32_t &w, uint32_t voff, const uint32_t *src)
{
    asm volatile("global_load_dword %0, %1, %2 sc1" : "=&v"(w) : "v"(voff), "s"(src) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// every wave's loads for the next phase have landed and every wave has left the phase before
template <int N> __device__ __forceinline__ void phase_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<N>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Waits until *flag == epoch; gives up after `limit` ticks of the 100 MHz wall clock (0: at once).
// (a rare path: an ordinary load, and the wait the compiler puts behind it drains everything)
__device__ __noinline__ bool wait_flag(const uint32_t *flag, uint32_t epoch, uint64_t limit)
{
    const uint64_t t0 = wall_clock64();
    for (;;) {
        if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == epoch) return true;
        if (wall_clock64() - t0 >= limit) return false;
        __builtin_amdgcn_s_sleep(8);
    }
}

// One pass over the chunks [c_begin, c_end) of one (sequence, head): 256 threads, kLds bytes at `lds`.
//   slot0, slot_stride   the slot of chunk c_begin and the byte distance to the next chunk's
//   ready                flag of chunk c_begin (consecutive chunks follow); epoch: value of a raised flag
//   st_base              element offset of this lane's column in the [d_k][d_v] states: pair * D * D + 32 c + x
//   poisoned             start from NaN instead of state_in (the caller could not obtain the initial state)
//   status               word that records a wait that ran out (the state is then poisoned with NaN, so
//                        every later output of this pass and its final state are NaN)
//   kGate, gate           the output gate of Section 4 applied to O before it is stored:
//                        o <- Sigmoid(g) * RMSNorm(o) * w, the mean square taken over the d_v values of a token
//                        (the four waves of the workgroup); gate.factors: w_j Sigmoid(g_tj) as fp16 in accumulator
//                        order, as the per-chunk role leaves them, kGateSlotBytes per chunk, this pair's first
//                        chunk of the pass
struct GateParams {
    const uint8_t *factors;
    float eps;
};
template <bool kFlags, bool kOutBf16, int kRole = kRoleFull, bool kGate = false>
__device__ __forceinline__ bool kda_scan4_body(uint8_t *lds, const uint8_t *slot0, int64_t slot_stride,
                                               const float *state_in, float *state_out, void *o, int64_t st_base,
                                               int64_t tok_base, int64_t len, int H, int64_t c_begin, int64_t c_end,
                                               int h, const uint32_t *ready, uint32_t epoch, uint32_t *status,
                                               uint64_t wait_limit, bool poisoned = false,
                                               const GateParams gate = GateParams{nullptr, 0.f})
{
    static_assert(!kGate || kRole == kRoleFull, "only a pass that writes outputs has a gate to apply");
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = __builtin_amdgcn_readfirstlane(tid >> 6);       // the wave: column slice of S, V_new, O
    // The chain of steps is the critical path of the whole prefill, the per-chunk workgroups that share the
    // compute unit are throughput work: the waves of this role go first where both want to issue.
    __builtin_amdgcn_s_setprio(3);
    const int x = lane & 31, hh = lane >> 5;
    const uint32_t lane16 = (uint32_t)lane * 16;
    constexpr bool kFull = kRole == kRoleFull;

    // vector-memory instructions per step, in issue order (see the loop)
    constexpr int nFlag = kFlags ? 1 : 0, nW = 4, nA = 2, nU = (kRole != kRoleT) ? 4 : 0;
    constexpr int nQ = kFull ? 4 : 0, nSt = kFull ? (kOutBf16 ? 4 : 8) : 0, nK = 4;
    constexpr int G0 = kGate ? 4 : 0;                             // the step's own gate factors, first thing in phase V
    constexpr int G1 = nFlag + nW + nA + nU, G2 = nQ, G3 = nSt, G4 = nK;

    // own state tiles in accumulator order: S[t][j] = S(dk = 32 t + acc_row(j, hh), dv = 32 c + x)
    f32x16 S[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int row = 32 * t + acc_row(j, hh);
            if (kRole == kRoleT)      S[t][j] = (row == 32 * c + x) ? 1.f : 0.f;
            else if (kRole == kRoleB) S[t][j] = 0.f;
            else                      S[t][j] = poisoned ? __builtin_nanf("") : (state_in ? state_in[st_base + (int64_t)row * D] : 0.f);
        }

    if (c_begin < c_end) {
        const uint32_t lds0 = (uint32_t)(uintptr_t)lds;          // LDS byte address of the ring
        const int64_t nsteps = c_end - c_begin;
        // this wave's share of a piece: fragments 4 c .. 4 c + 3 of a big one, 2 c, 2 c + 1 of a small one
        const uint32_t voff_big = lane16 + (uint32_t)c * 4096, voff_small = lane16 + (uint32_t)c * 2048;
        const uint32_t voff_u = lane16 + (uint32_t)c * kUTileBytes;
        // gate factors of this wave: tiles (P, c), P = 0, 1, two 16-byte units per lane and tile
        const uint32_t voff_g = lane16 + (uint32_t)c * kGateTileBytes;
        bool gave_up = false;
        auto gate_of = [&](int64_t rel) __attribute__((always_inline)) {       // clamped past the end
            return gate.factors + ((rel < nsteps) ? rel : nsteps - 1) * (int64_t)kGateSlotBytes;
        };

        auto slot_of = [&](int64_t rel) __attribute__((always_inline)) {       // clamped past the end
            return slot0 + ((rel < nsteps) ? rel : nsteps - 1) * slot_stride;
        };
        auto flag_of = [&](int64_t rel) __attribute__((always_inline)) {
            return ready + ((rel < nsteps) ? rel : nsteps - 1);
        };
        auto issue_w = [&](const uint8_t *slot, int region) __attribute__((always_inline)) {
            dma4(lds0 + (uint32_t)region * kBig + (uint32_t)c * 4096, voff_big, slot + kOffWn);
        };
        auto issue_q = [&](const uint8_t *slot, int region) __attribute__((always_inline)) {
            if (kFull) dma4(lds0 + (uint32_t)region * kBig + (uint32_t)c * 4096, voff_big, slot + kOffQp);
        };
        auto issue_k = [&](const uint8_t *slot, int region) __attribute__((always_inline)) {
            dma4(lds0 + (uint32_t)region * kBig + (uint32_t)c * 4096, voff_big, slot + kOffKt);
        };
        auto issue_a = [&](const uint8_t *slot, int small) __attribute__((always_inline)) {
            dma2(lds0 + kSmallRegions + (uint32_t)small * kSmall + (uint32_t)c * 2048, voff_small, slot + kOffAqk);
        };
        auto poison = [&]() __attribute__((always_inline)) {
            gave_up = true;
            if (lane == 0) __hip_atomic_fetch_or(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float bad = __builtin_nanf("");
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int j = 0; j < 16; ++j) S[t][j] = bad;
        };

        // ---- prologue: the whole first slot, waited for in full ----
        u32x4 ur[4];                                             // U tiles (0, c), (1, c): two 16-byte units each
        uint32_t seen = epoch;
        if (kFlags && !wait_flag(flag_of(0), epoch, wait_limit)) poison();
        {
            const uint8_t *s0 = slot_of(0);
            if (kFlags) load_word(seen, 0u, flag_of(1));
            issue_w(s0, 0);
            issue_a(s0, 0);
            if (kRole != kRoleT) {
                load2(ur[0], ur[1], voff_u, s0 + kOffU);
                load2(ur[2], ur[3], voff_u, s0 + kOffU + 4 * kUTileBytes);
            }
            issue_q(s0, 1);
            issue_k(s0, 2);
        }
        phase_barrier<0>();
        bool next_ok = !kFlags || (uint32_t)__builtin_amdgcn_readfirstlane((int)seen) == epoch;

        f32x16 av[2];                                            // V_new tiles (token tile P, columns of this wave)
        auto take_u = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int P = 0; P < 2; ++P)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int z = 0; z < 4; ++z) {
                        const uint32_t w2 = ur[2 * P + i][z];
                        const h2 pr = __builtin_bit_cast(h2, w2);
                        av[P][8 * i + 2 * z] = (kRole == kRoleT) ? 0.f : (float)pr[0];
                        av[P][8 * i + 2 * z + 1] = (kRole == kRoleT) ? 0.f : (float)pr[1];
                    }
        };
        take_u();

        const uint32_t o_rstride = (uint32_t)H * D * (kOutBf16 ? 2 : 4);   // bytes between consecutive tokens of o
        constexpr int LA = 4, RING = LA + 2;                     // operand fragments read ahead of the product that uses them
        // Vector-memory instructions are handed to the memory pipe one at a time between the matrix
        // products (a burst of them stalls the wave at issue, and the products behind it), in this order:
        //   phase V  (gate: the factors of this step, G0,) the flag of the step after next, then W, the small piece and
        //            U of the next step                                                                 (G1)
        //   phase O  Gamma.Q of the next step                                                          (G2)
        //   phase S  K^T of the next step (G4), then this step's output stores                         (G3)
        constexpr int kStores = nSt;

        for (int64_t rel = 0; rel < nsteps; ++rel) {
            // pieces of this step sit in regions rW (W), rQ (Gamma.Q), rK (K^T); the region after them takes W of the next step
            const int p3 = (int)((3 * rel) & 3);
            const int rW = p3, rQ = (p3 + 1) & 3, rK = (p3 + 2) & 3, rN = (p3 + 3) & 3;
            const int sm = (int)(rel & 1);
            const uint8_t *ldsW = lds + rW * kBig + lane16, *ldsQ = lds + rQ * kBig + lane16, *ldsK = lds + rK * kBig + lane16;
            const uint8_t *ldsA = lds + kSmallRegions + sm * kSmall + lane16;
            // (kGate: what depends on the lane number is formed afresh in every step: carried in registers across the loop
            // these were the values too many, and a reload from scratch memory waits for every load in flight, once per
            // step; a volatile statement, or the compiler forms them once ahead of the loop all the same)
            auto lane_now = [&]() __attribute__((always_inline)) {
                int l;
                asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
                return l;
            };
            const int hh_step = kGate ? (lane_now() >> 5) : hh;
            const float *gc = reinterpret_cast<const float *>(lds + kSmallRegions + sm * kSmall + (kOffGc - kOffAqk)) + 4 * hh_step;
            const uint8_t *nxt = slot_of(rel + 1);
            const uint8_t *gate_cur = kGate ? gate_of(rel) : nullptr;
            u32x4 gr[4];                                         // kGate: gate factors of tiles (0, c), (1, c), two 16-byte units each
            float *red = reinterpret_cast<float *>(lds + kSmallRegions + sm * kSmall + kGateRed);   // idle tail of the small region: kGate's partial mean squares, kRoleT's flags
            const uint32_t m0W = lds0 + (uint32_t)rN * kBig + (uint32_t)c * 4096;      // W of the next step
            const uint32_t m0Q = lds0 + (uint32_t)rW * kBig + (uint32_t)c * 4096;      // Gamma.Q of the next step (over this step's W)
            const uint32_t m0K = lds0 + (uint32_t)rQ * kBig + (uint32_t)c * 4096;      // K^T of the next step (over this step's Gamma.Q)
            const uint32_t m0A = lds0 + kSmallRegions + (uint32_t)(sm ^ 1) * kSmall + (uint32_t)c * 2048;

            if (kFlags && !next_ok && !gave_up) {
                if (!wait_flag(flag_of(rel + 1), epoch, wait_limit)) poison();
            }
            const uint32_t *flag2 = kFlags ? flag_of(rel + 2) : nullptr;
            __builtin_amdgcn_sched_barrier(0);

            // ---- phase V: V_new[P] = U[P] + (-W)(P, tau, s) S(tau, s), slot i: P = i % 2, (tau, s) = i / 2 ----
            h8 Sb[8];                                            // fp16 copy of S as it enters the step: (tau, s) -> Sb[2 tau + s]
            {
                h8 ring[RING];
                auto frag = [&](const int i) __attribute__((always_inline)) {
                    return *reinterpret_cast<const h8 *>(ldsW + frag_rts(i % 2, (i / 2) / 2, (i / 2) % 2) * kFragBytes);
                };
                static_for<0, LA>([&](auto ic) __attribute__((always_inline)) { ring[decltype(ic)::value % RING] = frag(decltype(ic)::value); });
                static_for<0, 16>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int i = decltype(ic)::value, P = i % 2, tau = (i / 2) / 2, s = (i / 2) % 2;
                    if constexpr (i + LA < 16) ring[(i + LA) % RING] = frag(i + LA);
                    if constexpr (P == 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) Sb[i / 2][e] = (_Float16)S[tau][8 * s + e];
                    }
                    av[P] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ring[i % RING], Sb[i / 2], av[P], 0, 0, 0);
                    // G0 (this step's gate factors), then G1, one instruction per slot
                    constexpr int j = i - G0;
                    if constexpr (i < G0) load1(gr[i], voff_g, gate_cur + (i / 2) * 4 * kGateTileBytes + (i % 2) * 1024);
                    else if constexpr (j == 0) { if (kFlags) load_word(seen, 0u, flag2); }
                    else if constexpr (j >= 1 && j <= 4) dma1(m0W + (j - 1) * 1024, voff_big, nxt + kOffWn + (j - 1) * 1024);
                    else if constexpr (j >= 5 && j <= 6) dma1(m0A + (j - 5) * 1024, voff_small, nxt + kOffAqk + (j - 5) * 1024);
                    else if constexpr (j >= 7 && j <= 10) {
                        if (kRole != kRoleT)
                            load1(ur[j - 7], voff_u, nxt + kOffU + ((j - 7) / 2) * 4 * kUTileBytes + ((j - 7) % 2) * 1024);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
            // fp16 copy of V_new: registers 8 s .. 8 s + 7 of a tile are its slots of K-step s as a B operand
            h8 Vb[2][2];
#pragma unroll
            for (int P = 0; P < 2; ++P)
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int e = 0; e < 8; ++e) Vb[P][s][e] = (_Float16)av[P][8 * s + e];
            phase_barrier<G3 + G4 + G0 + G1>();                  // Gamma.Q (and the small piece) of this step

            // ---- phase O: O^T[P] = S^T (Gamma.Q)(P)^T + V_new^T Tril(A_qk)(P, rho)^T; between the products the
            // state is scaled, S <- Diag(gamma^C) S (the products read the fp16 copy taken in phase V) ----
            f32x16 ao[2] = {{0.f}, {0.f}};
            auto scale_state = [&](const int t, const int q4) __attribute__((always_inline)) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(gc + 32 * t + 8 * q4);
#pragma unroll
                for (int z = 0; z < 4; ++z) S[t][4 * q4 + z] *= gv[z];
            };
            if constexpr (kFull) {
                h8 ring[RING];
                // slots 0..15: Gamma.Q (P, tau, s) as in phase V; 16..21: A_qk (0,0,s) (1,0,s) (1,1,s)
                auto frag = [&](const int i) __attribute__((always_inline)) {
                    if (i < 16) return *reinterpret_cast<const h8 *>(ldsQ + frag_rts(i % 2, (i / 2) / 2, (i / 2) % 2) * kFragBytes);
                    return *reinterpret_cast<const h8 *>(ldsA + (i - 16) * kFragBytes);
                };
                static_for<0, LA>([&](auto ic) __attribute__((always_inline)) { ring[decltype(ic)::value % RING] = frag(decltype(ic)::value); });
                static_for<0, 22>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int i = decltype(ic)::value;
                    if constexpr (i + LA < 22) ring[(i + LA) % RING] = frag(i + LA);
                    if constexpr (i < 16) {
                        constexpr int P = i % 2;
                        ao[P] = __builtin_amdgcn_mfma_f32_32x32x16_f16(Sb[i / 2], ring[i % RING], ao[P], 0, 0, 0);
                        scale_state(i / 4, i % 4);
                    } else {
                        // fragment (rr, ri, s) of Tril(A_qk): output token tile rr, V_new token tile ri
                        constexpr int j = i - 16, rr = (j < 2) ? 0 : 1, ri = (j < 4) ? 0 : 1, s = j % 2;
                        ao[rr] = __builtin_amdgcn_mfma_f32_32x32x16_f16(Vb[ri][s], ring[i % RING], ao[rr], 0, 0, 0);
                    }
                    if constexpr (i < 4) dma1(m0Q + i * 1024, voff_big, nxt + kOffQp + i * 1024);      // G2
                    __builtin_amdgcn_sched_barrier(0);
                });
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) scale_state(i / 4, i % 4);
            }
            if (kGate) {
                // A token's 128 outputs sit in two lanes of each of the four waves: lane-local sum of squares, the
                // two lanes by a swap, the four waves through the unused tail of this step's small region (the
                // barrier that ends the phase publishes it).
                const int ln = lane_now();
#pragma unroll
                for (int P = 0; P < 2; ++P) {
                    float ssq = 0.f;
#pragma unroll
                    for (int j = 0; j < 16; ++j) ssq = fmaf(ao[P][j], ao[P][j], ssq);
                    ssq += __shfl_xor(ssq, 32);
                    if (ln < 32) red[(P * 4 + c) * 32 + ln] = ssq;
                }
                // (the barrier below waits for vector memory only: the LDS stores above are waited for here)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            // O <- Sigmoid(g) * RMSNorm(O) * w on tile P, in place (phase S, before the tile is turned for the stores)
            auto apply_gate = [&](const int P) __attribute__((always_inline)) {
                const int xl = lane_now() & 31;
                const float tot = red[(P * 4 + 0) * 32 + xl] + red[(P * 4 + 1) * 32 + xl] + red[(P * 4 + 2) * 32 + xl] +
                                  red[(P * 4 + 3) * 32 + xl];
                const float rstd = __builtin_amdgcn_rsqf(tot * (1.0f / D) + gate.eps);
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int wd = 0; wd < 4; ++wd) {
                        // word wd of unit `half`: columns 32 c + 8 q4 + 4 hh + 2 w, + 1 with q4 = 2 half + wd / 2, w = wd % 2
                        // (through a scalar: a bit cast applied to a vector element directly reads element 0)
                        const uint32_t w2 = gr[2 * P + half][wd];
                        const h2 pr = __builtin_bit_cast(h2, w2);
                        const int idx = 4 * (2 * half + (wd >> 1)) + 2 * (wd & 1);
                        ao[P][idx] *= rstd * (float)pr[0];
                        ao[P][idx + 1] *= rstd * (float)pr[1];
                    }
            };
            // O^T accumulator: lane (token 32 P + x, hh), registers 4 q .. 4 q + 3 = columns 32 c + 8 q + 4 hh + 0..3:
            // a token's 128 bytes of this wave's columns sit in two lanes, 16 bytes per register group.  Stored
            // that way, one instruction touches 32 cache lines and every line is written four times over; the
            // memory pipe pays per line.  The four lanes of a quad therefore transpose their 4 x 4 register
            // groups (in phase S, between the products): afterwards lane (x, hh) holds group x % 4 of the tokens
            // 4 (x / 4) + 0..3, so that store i writes the whole line of token 4 (x / 4) + i from eight lanes:
            // eight lines per instruction, each once.
            u32x4 ot[2][4];
            auto prepare_out = [&](const int P, const int z) __attribute__((always_inline)) {
                if constexpr (!kOutBf16) {
                    float r[4] = {ao[P][z], ao[P][4 + z], ao[P][8 + z], ao[P][12 + z]};
                    quad_transpose(r, lane);
#pragma unroll
                    for (int i = 0; i < 4; ++i) ot[P][i][z] = __float_as_uint(r[i]);
                } else if (z == 0) {
                    // bf16: w[2 q4 + z] = columns 8 q4 + 4 hh + 2 z, + 1.  The two lanes of a token trade
                    // halves, so each ends up with two runs of eight consecutive columns: two stores.
                    uint32_t w[8];
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        w[2 * q4] = pack_bf16x2(ao[P][4 * q4], ao[P][4 * q4 + 1]);
                        w[2 * q4 + 1] = pack_bf16x2(ao[P][4 * q4 + 2], ao[P][4 * q4 + 3]);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(w[i], w[4 + i], false, false);
                        w[i] = sw[0]; w[4 + i] = sw[1];
                    }
#pragma unroll
                    for (int qq = 0; qq < 2; ++qq) {
                        u32x4 val = {w[2 * qq], w[2 * qq + 1], w[4 + 2 * qq], w[4 + 2 * qq + 1]};
                        ot[P][qq] = val;
                    }
                }
            };
            // The stores go through a buffer descriptor that covers the chunk's real tokens: rows of
            // tokens past the end of the sequence are dropped by the hardware, and the number of
            // store instructions does not depend on the data.
            const int64_t t0 = (c_begin + rel) * kChunk;
            const int64_t left = len - t0;
            const uint32_t nvalid = (uint32_t)(left < kChunk ? left : kChunk);
            uint8_t *obase = static_cast<uint8_t *>(o) + ((tok_base + t0) * H + h) * (int64_t)(D * (kOutBf16 ? 2 : 4));
            const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(obase, 0, (int)(nvalid * o_rstride), 0x00020000);
            // fp32: store i of tile P: token 32 P + 4 (x / 4) + i, columns 32 c + 8 (x % 4) + 4 hh + 0..3
            // bf16: store qq of tile P: token 32 P + x, columns 32 c + 8 (qq + 2 hh) + 0..7
            const uint32_t ol = kOutBf16 ? (uint32_t)x * o_rstride + (uint32_t)(32 * c + 16 * hh) * 2
                                         : (uint32_t)(x & ~3) * o_rstride + (uint32_t)(32 * c + 8 * (x & 3) + 4 * hh) * 4;
            // K^T of this step; with the gate also its factors, which were issued after the stores of the step before:
            // those stores are then waited for as well
            phase_barrier<kGate ? G1 + G2 : G1 + G2 + G3>();

            // ---- phase S: S += (Gamma^{i->C}.K)^T V_new (S is already scaled), slot i: tau = i % 4, (rho, s) = i / 4.
            // Slots 0..3 also issue K^T of the next step and turn output tile 0 into store order, 4..7 store it
            // and turn tile 1, 8..11 store tile 1 ----
            {
                h8 ring[RING];
                auto frag = [&](const int i) __attribute__((always_inline)) {
                    return *reinterpret_cast<const h8 *>(ldsK + frag_trs(i % 4, (i / 4) / 2, (i / 4) % 2) * kFragBytes);
                };
                static_for<0, LA>([&](auto ic) __attribute__((always_inline)) { ring[decltype(ic)::value % RING] = frag(decltype(ic)::value); });
                static_for<0, 16>([&](auto ic) __attribute__((always_inline)) {
                    constexpr int i = decltype(ic)::value, tau = i % 4, rho = (i / 4) / 2, s = (i / 4) % 2;
                    if constexpr (i + LA < 16) ring[(i + LA) % RING] = frag(i + LA);
                    S[tau] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ring[i % RING], Vb[rho][s], S[tau], 0, 0, 0);
                    if constexpr (i < 4) dma1(m0K + i * 1024, voff_big, nxt + kOffKt + i * 1024);      // G4
                    if constexpr (kGate && (i == 0 || i == 4)) apply_gate(i / 4);
                    if constexpr (kFull && i < 8) prepare_out(i / 4, i % 4);
                    if constexpr (kFull && i >= 4 && i < 12) {                                          // G3
                        constexpr int P = (i - 4) / 4, k = (i - 4) % 4;
                        if constexpr (k < kStores / 2) {
                            const uint32_t off = ol + (uint32_t)(32 * P) * o_rstride + (kOutBf16 ? (uint32_t)k * 16 : (uint32_t)k * o_rstride);
                            __builtin_amdgcn_raw_buffer_store_b128(ot[P][k], orsrc, (int)off, 0, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            }

            // kRoleT, every eighth step: has this wave's slice of the transition vanished, bit for bit?  Decay takes a
            // range's transition to exact zero within a few chunks (S is scaled by gamma^C every step and what the
            // products add is formed from it), and zero stays zero under every further step, so the rest of the range
            // need not be walked.  Every wave still loads its share of the operands for the others, so the four
            // waves leave together: flags through the idle tail of this step's small region.
            const bool probe = kRole == kRoleT && (rel & 7) == 7;
            if (probe) {
                uint32_t bits = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int j = 0; j < 16; ++j) bits |= __float_as_uint(S[t][j]);
                const bool zero = __builtin_amdgcn_ballot_w64((bits & 0x7fffffffu) != 0) == 0;
                if (lane == 0) reinterpret_cast<uint32_t *>(red)[c] = zero ? 1u : 0u;
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }

            // ---- the next step's W and U are here: take U, note whether the flag read in phase V was up ----
            phase_barrier<G2 + G3 + G4>();
            take_u();
            if (kFlags) next_ok = (uint32_t)__builtin_amdgcn_readfirstlane((int)seen) == epoch;
            if (probe) {
                const uint32_t *zf = reinterpret_cast<const uint32_t *>(red);
                const bool all_zero = (zf[0] & zf[1] & zf[2] & zf[3]) != 0;
                // (nobody's next loads may land on the flags before everybody has read them)
                __builtin_amdgcn_s_barrier();
                if (all_zero) break;                             // the same answer in every thread of the workgroup
            }
        }
        // the loads issued for a step that does not exist (clamped to the last slot) must not land after the
        // workgroup has given its LDS back
        wait_vm<0>();
    }

    // A state that is not finite at the end of the pass means that an fp16 operand overflowed on the way
    // (values outside the documented domain) or that a wait ran out: recorded as bit 1 of the status word.
    {
        bool bad = false;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j) bad |= !(__builtin_fabsf(S[t][j]) < __builtin_inff());
        if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0)
            __hip_atomic_fetch_or(status, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (state_out && (state_out != state_in || c_begin < c_end)) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                state_out[st_base + (int64_t)(32 * t + acc_row(j, hh)) * D] = S[t][j];
    }
    bool vanished = false;
    if (kRole == kRoleT) {
        // the transition as it stands at the end of the pass, whichever way the loop was left: all four slices zero?
        uint32_t bits = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j) bits |= __float_as_uint(S[t][j]);
        const bool zero = __builtin_amdgcn_ballot_w64((bits & 0x7fffffffu) != 0) == 0;
        volatile uint32_t *zf = reinterpret_cast<volatile uint32_t *>(lds);
        __syncthreads();                                         // nobody reads operands from the LDS any more
        if (lane == 0) zf[c] = zero ? 1u : 0u;
        __syncthreads();
        vanished = (zf[0] & zf[1] & zf[2] & zf[3]) != 0;
        __syncthreads();                                         // the words are free again
    }
    return vanished;
}

}  // namespace scan4
}  // namespace mfma
}  // namespace kda
