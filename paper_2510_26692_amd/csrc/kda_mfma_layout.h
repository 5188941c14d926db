// Workspace layout shared by the two kernels of the matrix-core prefill path.
//
// kda_intra (parallel over chunks) leaves, for every (chunk, head) "slot", the
// operands that the sequential kda_scan needs, already arranged in the register
// order of the 32x32x16 f16 MFMA so that kda_scan moves them with straight
// 16-byte copies and never transposes anything:
//
//   Wn   -W            A operand [token r][dk]      frags [rho][tau][s]      fp16
//   Qp   Gamma.Q       A operand [token r][dk]      frags [rho][tau][s]      fp16
//   Kt   (Gamma^{i->C}.K)^T  A operand [dk][token]  frags [tau][rho][s]      fp16
//   Aqk  Tril(A_qk)    A operand [token r][token i] frags (0,0,s) (1,0,s) (1,1,s) fp16
//   gC   gamma^C       [dk]                                                  fp32
//   U                  C/D tiles [rho][ct] in accumulator order              fp16
//
// rho: 32-token tile, tau: 32-channel d_k tile, ct: 32-column d_v tile, s: one
// K-step of 16.  A "frag" is 64 lanes x 8 halfs (1 KiB); lane L = (x = L % 32,
// hh = L / 32) holds row x of the tile and the 8 contraction slots e = 0..7 of
// K-step s, where slot (hh, e) stands for contraction index
//
//       kidx(s, hh, e) = 16 s + 8 (e / 4) + 4 hh + (e % 4)          (0..31)
//
// inside the 32-wide tile.  This is the order in which a 32x32 accumulator tile
// (register j of lane (x, hh) holds row 8 (j/4) + 4 hh + j%4, column x) turns
// into a B operand with no data movement: registers 8 s .. 8 s + 7 of a lane are
// exactly its 8 slots of K-step s.  The state S and the pseudo-value V_new live
// in accumulators and are fed back as B operands that way.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace kda {
namespace mfma {

constexpr int D = 128;                        // d_k = d_v of this path
constexpr int kFragBytes = 1024;

constexpr int kOffWn = 0;                     // 16 frags
constexpr int kOffQp = kOffWn + 16 * kFragBytes;
constexpr int kOffKt = kOffQp + 16 * kFragBytes;
constexpr int kOffAqk = kOffKt + 16 * kFragBytes;   // 6 frags: token tile (0,1) of Tril(A_qk) is zero
constexpr int kOffGc = kOffAqk + 6 * kFragBytes;
constexpr int kLdsBlockBytes = kOffGc + D * 4;      // what kda_scan stages through LDS
constexpr int kUTileBytes = 64 * 16 * 2;            // one 32x32 tile of U: 16 halfs per lane, two 16-byte units
constexpr int kOffU = kLdsBlockBytes;               // 8 tiles x 2 KiB
constexpr int kSlotBytes = kOffU + 8 * kUTileBytes; // 72192
// Output gate (fused epilogue): the gate logits of a chunk, bf16, in the accumulator order of the
// sequential kernel's O tiles: tile (rho, ct) = [2 units][64 lanes][16 B], lane (x, hh) holds the
// columns 32 ct + 8 q + 4 hh + 0..3 of token 32 rho + x, q = 0..3 (unit q / 2, bytes 8 (q % 2) ..).
constexpr int kGateTileBytes = 64 * 16 * 2;
constexpr int kGateSlotBytes = 8 * kGateTileBytes;  // 16384, one per workspace slot when the gate is on

static_assert(kLdsBlockBytes % 16 == 0, "LDS block must be a whole number of 16-byte units");
static_assert(kSlotBytes % 256 == 0, "slots must stay 256-byte aligned");

// Contraction index inside a 32-wide tile for K-step s, lane half hh, slot e.
__host__ __device__ constexpr int kidx(int s, int hh, int e) { return 16 * s + 8 * (e >> 2) + 4 * hh + (e & 3); }
// Row inside a 32x32 accumulator tile held by register j of a lane in half hh.
__host__ __device__ constexpr int acc_row(int j, int hh) { return 8 * (j >> 2) + 4 * hh + (j & 3); }

constexpr int frag_rts(int r, int t, int s) { return (r * 4 + t) * 2 + s; }   // Wn, Qp: [rho][tau][s]
constexpr int frag_trs(int t, int r, int s) { return (t * 2 + r) * 2 + s; }   // Kt: [tau][rho][s]
constexpr int frag_aqk(int rr, int ri, int s) { return (rr + ri) * 2 + s; }   // (0,0) (1,0) (1,1)

// Time-split scan: at most this many ranges per sequence, offered to calls with at most this many
// (sequence, head) pairs whose longest sequence has at least kSplitMinChunks chunks.  The more pairs, the
// fewer ranges: 2 ranges - 1 scan workgroups per pair must start side by side on half of a device's
// workgroup slots (512 on MI355X).  split_parts_cap is that limit; it also sizes the state arrays in the
// workspace, so it depends on the number of pairs and on the chunk indices of a time segment alone.
constexpr int kSplitMaxParts = 32;
constexpr int kSplitMaxPairs = 64;
constexpr int kSplitMinChunks = 24;
constexpr int split_parts_cap(long long pairs, long long chunks)
{
    long long p = pairs > 0 ? (256 / pairs + 1) / 2 : kSplitMaxParts;
    if (p > chunks / 7 + 1) p = chunks / 7 + 1;               // (a range has at least 8 chunks)
    return p > kSplitMaxParts ? kSplitMaxParts : p < 2 ? 2 : (int)p;
}
static_assert(split_parts_cap(1, 1 << 20) == 32 && split_parts_cap(4, 1 << 20) == 32 && split_parts_cap(8, 1 << 20) == 16 &&
              split_parts_cap(16, 1 << 20) == 8 && split_parts_cap(32, 1 << 20) == 4 && split_parts_cap(48, 1 << 20) == 3 && split_parts_cap(64, 1 << 20) == 2 &&
              split_parts_cap(2, 64) == 10, "ranges offered by number of pairs and chunks");
// Packed calls with several batches of pairs and at most this many sequences take their sequences longest first
// (kda_prefill_fused.hip); the order sits behind the status word.
constexpr int kMaxOrderedSeqs = 256;
constexpr size_t kStatusAreaBytes = 256 + (size_t)kMaxOrderedSeqs * 4;
constexpr int kSplitTail = 32;               // chunks at a range's end over which its transition is expected to vanish
constexpr int kSplitMinTail = 16;            // ranges shorter than this do not try
constexpr int kSplitFlagsPerPair = 4 * kSplitMaxParts;      // u32 words per pair, ahead of the states
constexpr size_t kSplitFlagBytes = (size_t)kSplitMaxPairs * kSplitFlagsPerPair * 4;
static_assert(kSplitFlagBytes % 1024 == 0, "the area is cleared in blocks of 256 words and keeps what follows aligned");

// Geometry of one launch pair: `seg_chunks` chunk indices of every sequence.
struct SegPlan {
    int64_t seg_chunks;      // chunks per sequence held in the workspace at once
    int64_t num_segments;    // passes over the time axis
    size_t slots_offset;     // first slot (the status word sits in front of it)
    size_t carry_offset;     // byte offset of the state carry buffer in the workspace
    size_t flags_offset;     // one u32 "slot ready" flag per (sequence, head, chunk of the segment)
    size_t status_offset;    // u32 set by kda_scan when a bounded wait for a flag ran out
    size_t gate_offset;      // staged gate logits, kGateSlotBytes per slot (0: no output gate)
    size_t split_offset;     // time-split scan: kSplitFlagBytes of counters, then E, T, B, each [split_parts_cap(pairs, seg_chunks)][pairs][128][128] fp32
    size_t total_bytes;
};

}  // namespace mfma
}  // namespace kda
