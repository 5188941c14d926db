// Time-split scan for few (sequence, head) pairs and long sequences, built from the four-wave scan
// (kda_scan4.h).  The chunk recurrence is affine in the state (Section 3.1: S_out = T S_in + B with T
// the product of the per-chunk transitions), so the chunk axis is cut into `parts` ranges, the first
// of `part0_len` chunk indices and the others of `part_len`, and 2 parts - 3 workgroups work on one
// pair side by side:
//   y = 0          scans range 0 from the initial state (outputs and all) and leaves its final state
//                  in E[0]; later it scans the last range from E[parts - 2] and delivers the final state.
//   y = 2 p - 1    computes the transition T_p of range p = 1 .. parts - 2; later it scans range p
//                  from E[p - 1].
//   y = 2 p        computes the offset B_p of range p.
// Between the phases, workgroups y = 1 .. workers form E[p] = T_p E[p-1] + B_p for p = 1 .. parts - 2,
// each on its own slice of the d_v columns (the columns do not interact).  Results travel through
// the workspace (E, Tm, Bm: arrays of [pairs][128][128] fp32 states, one per range) under per-pair
// counters: pf[p] = slices of E[p] that are complete (E[0]: set to `workers` at once), pf[8 + p] /
// pf[16 + p] = T_p / B_p complete.  Every producer makes its stores visible with a device-scope
// release before it raises the counter, every consumer follows its (bounded) wait with a
// device-scope acquire.  No first-phase work waits for anything but its slots, all these workgroups
// sit at the front of the grid and take well under half the device, so every wait ends.
#pragma once
#include "kda_prefill_fused.h"
#include "kda_scan4.h"

namespace kda {
namespace mfma {
namespace scan4 {

constexpr int kSplitFlagsPerPair = 24;


__device__ __forceinline__ int split_workers(int parts) { return (parts - 2 >= 4) ? 8 : (parts - 2 >= 2) ? 4 : 2; }

// E[p][:, col0 .. col0 + 16 CW) for p = 1 .. parts - 2, in fp32, by one 256-thread workgroup.
// Thread (ty, tx) owns rows 8 ty .. 8 ty + 7 and columns col0 + CW tx .. + CW - 1; the current
// slice of E sits in LDS.  All T_p and B_p are awaited first (they finish before E[0] does) and
// pulled into this die's L2; after that the chain crosses no fence: E[0] is read and E[p] written
// with device-scope accesses.  Returns false if a wait ran out.
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
            ok = wait_flag(pf + 8 + p, 1u, wait_limit) && wait_flag(pf + 16 + p, 1u, wait_limit);
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
// [0, 2 parts - 3).  nchunks: chunk indices of this pair inside the launch's time segment; ws_pair / ready_pair:
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
    const int kind = (y == 0) ? kRoleFull : ((y & 1) ? kRoleT : kRoleB);
    const int mid = (y + 1) / 2;                              // the range of the first phase
    const int workers = split_workers(parts);
    uint32_t *pf = sp.flags + pair * kSplitFlagsPerPair;
    const int64_t st_base = pair_base + 32 * wave + (lane & 31);
    volatile int &second_ok = *reinterpret_cast<volatile int *>(lds + kLds - 16);

#define KDA_SCAN4_PART(ROLE)                                                                                        \
    kda_scan4_body<true, kOutBf16, ROLE>(lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, state_in, \
                                         state_out, o, st_base, tok_base, len, H, cbase + c_begin, cbase + c_end, h,  \
                                         ready_pair + c_begin, epoch, status, wait_limit)
    {   // first phase: the own range, from the initial state / the identity / zero
        const float *state_in = (y == 0) ? h0 : nullptr;
        float *state_out = (y == 0) ? sp.E : (kind == kRoleT ? sp.Tm : sp.Bm) + mid * pair_states;
        int64_t c_begin = (mid == 0) ? 0 : sp.part0_len + (mid - 1) * sp.part_len;
        int64_t c_end = c_begin + ((mid == 0) ? sp.part0_len : sp.part_len);
        if (c_begin > nchunks) c_begin = nchunks;
        if (c_end > nchunks) c_end = nchunks;
        if (kind == kRoleFull)
            kda_scan4_body<true, kOutBf16, kRoleFull, kGate>(
                lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, state_in, state_out, o, st_base, tok_base,
                len, H, cbase + c_begin, cbase + c_end, h, ready_pair + c_begin, epoch, status, wait_limit, false,
                GateParams{kGate ? gate_pair + c_begin * (int64_t)kGateSlotBytes : nullptr, gate_eps});
        else if (kind == kRoleT) KDA_SCAN4_PART(kRoleT);
        else KDA_SCAN4_PART(kRoleB);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t *f = (kind == kRoleFull) ? pf : (kind == kRoleT) ? pf + 8 + mid : pf + 16 + mid;
            __hip_atomic_store(f, (kind == kRoleFull) ? (uint32_t)workers : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (y >= 1 && y <= workers) {
        float *sE = reinterpret_cast<float *>(lds);
        const int w = y - 1;
        bool ok;
        if (workers == 8)      ok = fold_slices<1>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 16 * w, parts, workers, pf, wait_limit);
        else if (workers == 4) ok = fold_slices<2>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 32 * w, parts, workers, pf, wait_limit);
        else                   ok = fold_slices<4>(sE, sp.E, sp.Tm, sp.Bm, pair_states, pair_base, 64 * w, parts, workers, pf, wait_limit);
        if (!ok && threadIdx.x == 0) __hip_atomic_fetch_or(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (kind == kRoleB) return;
    {   // second phase: the scan of a range whose initial state is now known
        const int part = (y == 0) ? parts - 1 : mid;
        const float *state_in = sp.E + (part - 1) * pair_states;
        float *state_out = (y == 0) ? state_final : nullptr;
        if (threadIdx.x == 0) {
            const bool ok = wait_flag(pf + part - 1, (uint32_t)workers, wait_limit);
            if (!ok) __hip_atomic_fetch_or(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            second_ok = ok;
        }
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        int64_t c_begin = sp.part0_len + (part - 1) * sp.part_len, c_end = c_begin + sp.part_len;   // part >= 1 here
        if (c_begin > nchunks) c_begin = nchunks;
        if (c_end > nchunks) c_end = nchunks;
        // (if the range's initial state never arrived, the scan starts from NaN: see kda_scan4_body's `poisoned`)
        const bool poisoned = second_ok == 0;
        if (poisoned) state_in = nullptr;
        kda_scan4_body<true, kOutBf16, kRoleFull, kGate>(
            lds, ws_pair + c_begin * (int64_t)kSlotBytes, (int64_t)kSlotBytes, state_in, state_out, o, st_base, tok_base, len, H,
            cbase + c_begin, cbase + c_end, h, ready_pair + c_begin, epoch, status, wait_limit, poisoned,
            GateParams{kGate ? gate_pair + c_begin * (int64_t)kGateSlotBytes : nullptr, gate_eps});
    }
#undef KDA_SCAN4_PART
}

}  // namespace scan4
}  // namespace mfma
}  // namespace kda
