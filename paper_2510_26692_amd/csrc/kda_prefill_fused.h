// Launch interface of the one-kernel prefill (kda_prefill_fused.hip).
#pragma once
#include "kda_intra.h"

namespace kda {
namespace mfma {

// (sequence, head) pairs per batch of the grid: the scan workgroups of a batch wait for the per-chunk
// workgroups behind them, and about two batches' worth of them are resident at a time, each on half a
// compute unit.  128 scan workgroups in flight is where an MI355X does best (64 cannot take the slots as fast
// as the per-chunk role makes them, 256 leave that role too little of the device); a device with fewer compute
// units gets batches of a quarter of its workgroup slots, so that two batches never take more than half.
constexpr int kMaxBatchPairs = 128;

// Chunks one workgroup of the per-chunk role works through (the fetch of each hides behind the one before).
constexpr int kItemsPerWorkgroup = 4;

// Time-split scan (kda_scan4_split.h): workspace areas and the cut of the chunk axis.
struct SplitArgs {
    float *E, *Tm, *Bm;          // [split_parts_cap(pairs, seg_chunks)][pairs][128][128] fp32 each
    uint32_t *flags;             // kSplitFlagsPerPair words per pair
    int64_t part_len, part0_len; // chunk indices of the first range and of every other one
    int64_t tail;                // chunks at the end of a range whose transition is tested for zero (<= both lengths)
    int parts;                   // 1: no time split
};

struct FusedArgs {
    const uint16_t *q, *k, *v, *log_alpha, *beta;
    const int32_t *cu;              // cu_seqlens or NULL
    const int32_t *order;           // packed calls in several batches: the sequences, longest first (NULL: as they come)
    const float *state_in;          // [N,H,dk,dv] or NULL (= zeros)
    float *state_out;               // [N,H,dk,dv] or NULL
    void *o;
    uint8_t *ws;                    // first slot of the segment
    uint32_t *ready;                // one flag per slot
    uint32_t *status;
    int64_t T;                      // tokens per batch row (fixed-length batches)
    int64_t pairs;                  // num_seqs * heads
    int64_t seg_chunks, seg_index;  // chunk indices per time segment, and which segment this launch works on
    int64_t launch_chunks;          // chunk indices this launch covers (<= seg_chunks)
    uint64_t wait_limit;            // ticks of the 100 MHz wall clock a scan workgroup waits for one slot
    int H, nb;
    float scale;
    uint32_t epoch;                 // value of a raised flag
    int producers;                  // 0: the per-chunk role does nothing (a diagnostic: every wait of the scan role then runs out)
    int per_wg, window;             // per-chunk role: chunks per workgroup, and workgroups that share a run of window * per_wg chunks
    RawParams raw;
    SplitArgs split;
    // output gate of Section 4 (kGate kernels only): o <- Sigmoid(g) * RMSNorm(o) * w
    const uint16_t *out_gate;       // gate logits [B,T,H,dv] bf16
    uint8_t *gate_ws;               // the same re-laid by the per-chunk role, kGateSlotBytes per slot
    const float *norm_w;            // [dv] or NULL (= ones)
    float rms_eps;
};

struct FusedLaunch {
    FusedArgs args;
    bool raw, scalar_gate, out_bf16, gate;
    bool reset_flags;               // clear num_flags words at args.ready and the status word first
    int64_t num_flags;
    int32_t *order_out;             // the first launch of such a call (the one that resets the flags) writes the order here, else NULL
    int num_seqs;
    bool reset_split;               // clear the counters of the time-split scan first (segments after the first)
    int compute_units;              // of the device the launch goes to
};

int fused_batch_pairs(int64_t pairs, int compute_units);
kda_status launch_prefill_fused(const FusedLaunch &L, hipStream_t stream);

}  // namespace mfma
}  // namespace kda
