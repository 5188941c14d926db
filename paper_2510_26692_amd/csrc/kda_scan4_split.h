// Time-split scan for few (sequence, head) pairs and long sequences, built from the four-wave scan
// (kda_scan4.h).  The chunk axis is cut into `parts` ranges, the first of `part0_len` chunk indices and
// the others of `part_len`, and the ranges of one pair are scanned side by side, each by a workgroup of
// its own.  What a range needs is the state at its start, E[p] = the state at the end of range p.
//
// The short way.  The chunk recurrence is affine in the state (Section 3.1: S_out = T S_in + B, T the
// product of the per-chunk transitions), and every step scales the state by the chunk's decay, so over
// enough chunks T vanishes: in fp32, bit for bit.  Where the transition of the last `tail` chunks of
// range p is exactly zero, the state at the end of the range does not depend on the state the range
// started from, and E[p] is the offset B of those chunks alone: `tail` steps from a zero state instead
// of the whole range.  Per pair, 2 parts - 1 workgroups:
//   y = 0          scans range 0 from the initial state (outputs and all) and leaves its final state in E[0].
//   y = 2 p + 1    forms the transition of the tail of range p, p = 0 .. parts - 2, and publishes the verdict:
//                  V[p] = 2 (zero) or 1 (not zero).  Then it scans range p + 1 from the offset of that tail;
//                  the last range delivers the final state.
//   y = 2 p + 2    forms the offset of the tail of range p (Bm[p]) and leaves.
// All ranges are under way after about `tail` steps, and the chain is one range long.
//
// The general way, for a pair in which some verdict is 1 (slow decay, or a sequence that ends before
// its ranges do): as soon as the verdicts are in, the same workgroups form the whole-range transitions and
// offsets and chain the range states through them,
//   y = 2 p + 1    T_p of range p = 1 .. parts - 2 into Tm[p]; later it scans range p from E[p - 1]
//                  (p = 0: nothing first, later the last range from E[parts - 2] and the final state),
//   y = 2 p + 2    B_p of range p = 1 .. parts - 2 into Bm[p],
//   y = 1 .. workers   then form E[p] = T_p E[p-1] + B_p for p = 1 .. parts - 2, each on its own slice of
//                  the d_v columns (the columns do not interact).
// which takes two ranges' time instead of one.  With tail = 0 (ranges too short for a transition to vanish)
// the tails are not tried and every pair goes this way at once.  A workgroup that cannot read the pair's verdicts
// (a bounded wait ran out) takes neither way: it reports the failure and writes NaN over the outputs it would
// have scanned on either.
//
// Results travel through the workspace (E, Tm, Bm: arrays of [pairs][128][128] fp32 states, one per
// range) under per-pair words: pf[p] = slices of E[p] that are complete (E[0]: set to `workers` at
// once), pf[kPfT + p] = T_p complete, pf[kPfB + p] = 1 when the tail's offset is in Bm[p], 2 when B_p
// is, pf[kPfV + p] = V[p].  Every producer makes its stores visible with a device-scope release before it
// raises a word, every consumer follows its (bounded) wait with a device-scope acquire.  No first
// pass waits for anything but its slots, all these workgroups sit at the front of the grid and take
// at most half the device, so every wait ends.
#pragma once
#include "kda_prefill_fused.h"
#include "kda_scan4.h"

namespace kda {
namespace mfma {
namespace scan4 {

// per-pair words: four groups of kSplitMaxParts
constexpr int kPfT = kSplitMaxParts, kPfB = 2 * kSplitMaxParts, kPfV = 3 * kSplitMaxParts;

__device__ __forceinline__ int split_workers(int parts) { return (parts - 2 >= 4) ? 8 : (parts - 2 >= 2) ? 4 : 2; }

// Waits until *flag is not zero and returns it; 0 after `limit` ticks of the 100 MHz wall clock.
__device__ __noinline__ uint32_t wait_nonzero(const uint32_t *flag, uint64_t limit)
{
    const uint64_t t0 = wall_clock64();
    for (;;) {
        const uint32_t v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v != 0) return v;
        if (wall_clock64() - t0 >= limit) return 0;
        __builtin_amdgcn_s_sleep(8);
    }
}

// NaN into the outputs of head h for the tokens [t_begin, t_end) of a sequence (clipped to its length): by 256 threads.
template <bool kOutBf16>
__device__ __forceinline__ void fill_nan(void *o, int64_t tok_base, int64_t len, int H, int h, int64_t t_begin, int64_t t_end)
{
    if (t_end > len) t_end = len;
    for (int64_t i = t_begin * D + threadIdx.x; i < t_end * D; i += 256) {
        const int64_t at = ((tok_base + i / D) * H + h) * (int64_t)D + i % D;
        if (kOutBf16) static_cast<uint16_t *>(o)[at] = 0x7fc0u;
        else          static_cast<float *>(o)[at] = __builtin_nanf("");
    }
}

// E[p][:, col0 .. col0 + 16 CW) for p = 1 .. parts - 2, in fp32, by one 256-thread workgroup.
// Thread (ty, tx) owns rows 8 ty .. 8 ty + 7 and columns col0 + CW tx .. + CW - 1; the current
// slice of E sits in LDS.  All T_p and B_p are awaited first (they are done at about the time E[0]
// is) and pulled into this die's L2; after that the chain crosses no fence: E[0] is read and E[p]
// written with device-scope accesses.  Returns false if a wait ran out.
template <int CW>
__device__ __forceinline__ bool fold_slices(float *sE, float *E, const float *Tm, const float *Bm, int64_t pair_states,
                                            int64_t pair_base, int col0, int parts, int workers, uint32_t *pf,
                                            uint64_t wait_limit)
{
    constexpr int NC = 16 * CW, NT = 256, RPT = D / (NT / 16);
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    // (a word at the very end of the workgroup's LDS, past everything the fold and the scan's first loads touch)
    volatile int &ok_word = *reinterpret_cast<volatile int *>(reinterpret_cast<uint8_t *>(sE) + kLds - 16);
    if (tid == 0) {
        bool ok = true;
        for (int p = 1; p <= parts - 2 && ok; ++p)
            ok = wait_flag(pf + kPfT + p, 1u, wait_limit) && wait_flag(pf + kPfB + p, 2u, wait_limit);
        ok_word = ok;
    }
    __syncthreads();
    bool ok = ok_word != 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    if (ok) {
        f32x4 touch = {0.f, 0.f, 0.f, 0.f};
        for (int p = 1; p <= parts - 2; ++p)
            for (int i = tid; i < D * D / 4; i += NT)
                touch += *reinterpret_cast<const f32x4 *>(Tm + p * pair_states + pair_base + 4 * i);
        asm volatile("" ::"v"(touch));
    }
    __syncthreads();
    if (tid == 0) ok_word = ok && wait_flag(pf, (uint32_t)workers, wait_limit);
    __syncthreads();
    ok = ok_word != 0;
    for (int i = tid; i < D * NC; i += NT)
        sE[i] = __hip_atomic_load(E + pair_base + (int64_t)(i / NC) * D + col0 + (i % NC), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    for (int p = 1; p <= parts - 2; ++p) {
        const float *Tp = Tm + p * pair_states + pair_base;
        const float *Bp = Bm + p * pair_states + pair_base + col0 + CW * tx;
        float acc[RPT][CW];
#pragma unroll
        for (int i = 0; i < RPT; ++i)
#pragma unroll
            for (int z = 0; z < CW; ++z) acc[i][z] = Bp[(int64_t)(RPT * ty + i) * D + z];
        for (int k4 = 0; k4 < D / 4; ++k4) {
            f32x4 a[RPT];
            float b[4][CW];
#pragma unroll
            for (int i = 0; i < RPT; ++i) a[i] = *reinterpret_cast<const f32x4 *>(Tp + (int64_t)(RPT * ty + i) * D + 4 * k4);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int z = 0; z < CW; ++z) b[kk][z] = sE[(4 * k4 + kk) * NC + CW * tx + z];
#pragma unroll
            for (int i = 0; i < RPT; ++i)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int z = 0; z < CW; ++z) acc[i][z] = fmaf(a[i][kk], b[kk][z], acc[i][z]);
        }
        __syncthreads();                                     // every thread is done reading the old slice
        float *Ep = E + p * pair_states + pair_base + col0 + CW * tx;
#pragma unroll
        for (int i = 0; i < RPT; ++i)
#pragma unroll
            for (int z = 0; z < CW; ++z) {
                // (a range state that could not be formed poisons everything scanned from it)
                const float val = ok ? acc[i][z] : __builtin_nanf("");
                sE[(RPT * ty + i) * NC + CW * tx + z] = val;
                __hip_atomic_store(Ep + (int64_t)(RPT * ty + i) * D + z, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): the write-through stores have landed
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(pf + p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return ok;
}

// One workgroup (256 threads) of the time-split scan: pair `pair` (sequence n, head h), role index y in
// [0, 2 parts - 1).  nchunks: chunk indices of this pair inside the launch's time segment; ws_pair / ready_pair:
// the pair's first slot and flag in the segment; cbase: the segment's first chunk index in the sequence.
// kGate: the passes that write outputs apply the output gate; gate_pair: the pair's first slot of gate factors, eps: of
// the RMSNorm (see kda_scan4_body).
template <bool kOutBf16, bool kGate = false>
__device__ __forceinline__ void split_role(uint8_t *lds, const SplitArgs &sp, const uint8_t *ws_pair, const uint32_t *ready_pair,
                                           const float *h0, float *state_final, void *o, int64_t pair, int64_t pairs, int y,
                                           int64_t tok_base, int64_t len, int H, int h, int64_t cbase, int64_t nchunks,
                                           uint32_t epoch, uint32_t *status, uint64_t wait_limit,
                                           const uint8_t *gate_pair = nullptr, float gate_eps = 0.f)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int parts = sp.parts;
    const int64_t pair_states = pairs * (int64_t)(D * D), pair_base = pair * (int64_t)(D * D);
    const int workers = split_workers(parts);
    uint32_t *pf = sp.flags + pair * kSplitFlagsPerPair;
    const int64_t st_base = pair_base + 32 * wave + (lane & 31);
    // (a word at the very end of the workgroup's LDS, past everything the scan's first loads touch)
    volatile int &word = *reinterpret_cast<volatile int *>(lds + kLds - 16);
    auto clip = [&](int64_t c) __attribute__((always_inline)) { return c < nchunks ? c : nchunks; };
    auto begin_of = [&](int r) __attribute__((always_inline)) { return r == 0 ? (int64_t)0 : sp.part0_len + (r - 1) * sp.part_len; };
    auto end_of = [&](int r) __attribute__((always_inline)) { return sp.part0_len + r * sp.part_len; };
    auto give_up = [&]() __attribute__((always_inline)) {
        __hip_atomic_fetch_or(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };

    // the scan of one range (outputs and all); every workgroup that scans comes through this one call
    int range;                       // the range to scan
    const float *state_in;           // its initial state
    bool poisoned = false;           // .. which never arrived
    if (y == 0) {
        range = 0; state_in = h0;
    } else {
        const int p = (y - 1) >> 1;                               // the boundary: end of range p
        const bool is_t = (y & 1) != 0;
        // ---- the tail of range p: transition (is it zero?) / offset; tail = 0: the host saw no point in trying ----
        int64_t c_begin = 0, c_end = 0;
        int way = sp.tail == 0 ? 1 : 0;                          // 0: short, 1: general, 2: unknown
        if (way == 1 && y == 1 && threadIdx.x == 0) __hip_atomic_fetch_or(status, 512u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma nounroll
        for (int pass = way; pass < 2; ++pass) {
            if (pass == 0) {
                c_end = end_of(p); c_begin = c_end - sp.tail;    // (tail <= every range's length)
            } else {
                if (p == 0) break;
                c_begin = begin_of(p); c_end = end_of(p);
            }
            c_begin = clip(c_begin); c_end = clip(c_end);
            // pass 0: the tail; pass 1 (general way, middle ranges only): the whole range
            float *state_out = is_t ? (pass ? sp.Tm + p * pair_states : nullptr) : sp.Bm + p * pair_states;
            bool vanished = false;
            if (is_t)
                vanished = kda_scan4_body<true, kOutBf16, kRoleT>(
                    lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, nullptr, state_out, o, st_base, tok_base,
                    len, H, cbase + c_begin, cbase + c_end, h, ready_pair + c_begin, epoch, status, wait_limit);
            else
                kda_scan4_body<true, kOutBf16, kRoleB>(
                    lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, nullptr, state_out, o, st_base, tok_base,
                    len, H, cbase + c_begin, cbase + c_end, h, ready_pair + c_begin, epoch, status, wait_limit);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __syncthreads();
            if (pass == 1) {
                if (threadIdx.x == 0)
                    __hip_atomic_store(is_t ? pf + kPfT + p : pf + kPfB + p, is_t ? 1u : 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            if (threadIdx.x == 0) {
                __hip_atomic_store(is_t ? pf + kPfV + p : pf + kPfB + p, is_t ? (vanished ? 2u : 1u) : 1u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                // The verdicts of all boundaries of the pair: they are written once, so all workgroups of the pair
                // that get to read them take the same way; one that does not (a wait ran out) takes neither.
                bool all_zero = true, all_seen = true;
                for (int b = 0; b <= parts - 2; ++b) {
                    const uint32_t v = wait_nonzero(pf + kPfV + b, wait_limit);
                    all_seen = all_seen && v != 0;
                    all_zero = all_zero && v == 2u;
                }
                if (!all_seen) give_up();
                word = !all_seen ? 2 : all_zero ? 0 : 1;
                // (for tests and measurement: which way pairs took, in two bits of the status word that report no failure)
                if (y == 1 && all_seen) __hip_atomic_fetch_or(status, all_zero ? 256u : 512u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            way = uni(word);                                     // (the same in every lane: branches and addresses stay scalar)
            __syncthreads();
            if (way != 1) break;
        }
        if (way == 2) {
            // Neither way can be taken.  Whatever this workgroup would have scanned on either is written as NaN (a
            // workgroup of the pair that did read the verdicts may write the true values over some of it: the
            // failure is in the status word, and no output keeps what the caller's buffer held before).
            if (!is_t) return;
            const int other = (p == 0) ? parts - 1 : p;
            fill_nan<kOutBf16>(o, tok_base, len, H, h, (cbase + clip(begin_of(p + 1))) * kChunk, (cbase + clip(end_of(p + 1))) * kChunk);
            fill_nan<kOutBf16>(o, tok_base, len, H, h, (cbase + clip(begin_of(other))) * kChunk, (cbase + clip(end_of(other))) * kChunk);
            if ((p + 1 == parts - 1 || other == parts - 1) && state_final != nullptr)
                for (int i = threadIdx.x; i < D * D; i += 256) state_final[pair_base + i] = __builtin_nanf("");
            return;
        } else if (way == 0) {
            if (!is_t) return;
            // the short way: range p + 1 starts from the offset of the tail of range p
            if (threadIdx.x == 0) {
                const bool ok = wait_flag(pf + kPfB + p, 1u, wait_limit);
                if (!ok) give_up();
                word = ok;
            }
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            poisoned = uni(word) == 0;
            range = p + 1; state_in = sp.Bm + p * pair_states;
        } else {
            if (y <= workers) {
                float *sE = reinterpret_cast<float *>(lds);
                const int w = y - 1;
                bool ok;
                if (workers == 8)      ok = fold_slices<1>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 16 * w, parts, workers, pf, wait_limit);
                else if (workers == 4) ok = fold_slices<2>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 32 * w, parts, workers, pf, wait_limit);
                else                   ok = fold_slices<4>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 64 * w, parts, workers, pf, wait_limit);
                if (!ok && threadIdx.x == 0) give_up();
                __syncthreads();
            }
            if (!is_t) return;
            // the general way: range p from E[p - 1]; the workgroup of boundary 0 takes the last range
            range = (p == 0) ? parts - 1 : p;
            if (threadIdx.x == 0) {
                const bool ok = wait_flag(pf + range - 1, (uint32_t)workers, wait_limit);
                if (!ok) give_up();
                word = ok;
            }
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            poisoned = uni(word) == 0;
            state_in = sp.E + (range - 1) * pair_states;
        }
        __syncthreads();
    }

    // (if the range's initial state never arrived, the scan starts from NaN: see kda_scan4_body's `poisoned`)
    if (poisoned) state_in = nullptr;
    // The last range delivers the final state.  Where that is the array the initial state was read from (a later time
    // segment of a call), the workgroup of range 0 may not have read it yet: the state then rests in E[parts - 1]
    // until that workgroup is done.
    const bool last = range == parts - 1;
    const bool detour = last && state_final != nullptr && state_final == h0;
    float *state_out = (range == 0) ? sp.E : last ? (detour ? sp.E + (int64_t)(parts - 1) * pair_states : state_final) : nullptr;
    const int64_t c_begin = clip(begin_of(range)), c_end = clip(end_of(range));
    kda_scan4_body<true, kOutBf16, kRoleFull, kGate>(
        lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, state_in, state_out, o, st_base, tok_base, len, H,
        cbase + c_begin, cbase + c_end, h, ready_pair + c_begin, epoch, status, wait_limit, poisoned,
        GateParams{kGate ? gate_pair + c_begin * (int64_t)kGateSlotBytes : nullptr, gate_eps});
    if (range == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (threadIdx.x == 0) __hip_atomic_store(pf, (uint32_t)workers, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (detour) {
        __syncthreads();
        if (threadIdx.x == 0) {
            const bool ok = wait_flag(pf, (uint32_t)workers, wait_limit);
            if (!ok) give_up();
            word = ok;
        }
        __syncthreads();
        const bool ok = uni(word) != 0;
        // (every thread moves the elements it has just written itself)
        const float *from = sp.E + (int64_t)(parts - 1) * pair_states;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int64_t at = st_base + (int64_t)(32 * t + acc_row(j, lane >> 5)) * D;
                state_final[at] = ok ? from[at] : __builtin_nanf("");
            }
    }
}

}  // namespace scan4
}  // namespace mfma
}  // namespace kda
