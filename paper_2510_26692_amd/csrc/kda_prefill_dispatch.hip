// Host side of the matrix-core prefill (bf16 inputs, d_k = d_v = 128, C = 64): workspace plan, the
// decision whether to cut the chunk axis into ranges, and the launches.  No kernel lives here; the
// device code is in kda_prefill_fused.hip.
//
// Nothing is allocated, no stream or event is created and the host never waits: a call is one launch
// per time segment on the caller's stream (plus a small fill kernel for the flags).
#include <stdlib.h>

#include "kda_prefill_fused.h"

namespace kda {

extern int g_split;            // diagnostics switches owned by kda_api.hip (see kda_debug.h)
extern double g_split_ratio;
extern int g_split_tail;
extern int g_producers;
extern uint64_t g_wait_limit;

namespace mfma {

__global__ void kda_zero_words_kernel(uint32_t *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

static int64_t max_chunks_per_seq(const kda_dims *d)
{
    int64_t longest = d->seqlen;
    if (d->num_seqs != d->batch || d->batch == 1) {           // packed (or a single row)
        if (d->max_seqlen > 0 && d->max_seqlen < longest) longest = d->max_seqlen;
    }
    return (longest + kChunk - 1) / kChunk;
}

static size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace: [status word, 256 B; sequence order, 1 KiB][slots of one segment, pair by pair][state carry][ready flags, one per slot]
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
    p.slots_offset = kStatusAreaBytes;
    p.carry_offset = p.slots_offset + (size_t)sc * streams * kSlotBytes;
    p.flags_offset = p.carry_offset + carry;
    p.split_offset = round_up(p.flags_offset + (size_t)sc * streams * sizeof(uint32_t), 256);
    // counters and states of the time-split scan, when the call qualifies for it
    const bool split = streams <= (size_t)kSplitMaxPairs && sc >= kSplitMinChunks;
    p.total_bytes = p.split_offset + (split ? kSplitFlagBytes + 3 * (size_t)split_parts_cap((long long)streams, sc) * carry : 0);
    p.gate_offset = 0;
    if (gate) {
        p.gate_offset = round_up(p.total_bytes, 256);
        p.total_bytes = p.gate_offset + (size_t)sc * streams * kGateSlotBytes;
    }
    return p;
}

// How the time-split scan cuts a segment's chunk axis: parts = 1 means the plain scan.
struct SplitCut {
    int parts;
    int64_t part0_len, part_len;   // chunk indices of the first range and of each other one
    int64_t tail;                  // chunks at a range's end tested for a vanished transition; 0: not tried
};

// Every workgroup of either stage takes half a compute unit; a split launch starts 2 parts - 1 scan
// workgroups per pair, at most half of all slots, of which `parts` per pair stay for the length of a
// range on the short way (the others leave after the tail of one), at most three eighths of all
// slots, so that the per-chunk stage, the larger half of the work, keeps the rest.  Among the
// admissible numbers of ranges the one with the smallest estimated duration is taken, the plain scan
// included.  The estimates are in microseconds, fitted to measurements on MI355X with both stages
// sharing the compute units; a step of the scan takes 3.0.  (Two ranges are offered up to 64 pairs: what
// they buy there is not a shorter chain but twice the scan workgroups, whose steps, not the per-chunk
// stage, pace a long call of 64 pairs.)
//   Ranges of at least kSplitMinTail chunks try the short way: the tails (half a range, within
// kSplitMinTail .. kSplitTail chunks) are produced and walked first, then all ranges go side by side.
// With all slots busy a chunk of the per-chunk stage costs 21.2 on one slot, and a scan workgroup,
// which mostly waits, takes a quarter of a slot from that stage.  The per-chunk stage sets the pace as
// long as the chain of scan steps stays under half its time; a longer chain falls behind now and then
// and finishes up to a quarter later (fitted), and a chain longer than that is the duration.  Half the
// time the tails take to produce comes on top.  (The host cannot know whether the data lets the
// transitions vanish; the estimate assumes it does.)
//   Shorter ranges leave no room for a transition to vanish and take the general way at once: two
// phases, the first range shorter by the ratio of a pass that writes no output to the full scan (0.7)
// when the scan, not the per-chunk stage, sets the pace of the first phase; a chunk of the per-chunk
// stage 17 on one slot of a device that is not full, the fold and the extra start-up 60 + 12 per
// middle range.
// forced = 2..32: the largest admissible number up to `forced`, whatever the estimate says.
static SplitCut split_cut(const SegPlan &plan, const kda_dims *d, int cus, int forced)
{
    SplitCut cut = {1, 0, 0, 0};
    int64_t maxc = max_chunks_per_seq(d);                    // chunks one launch walks
    if (maxc > plan.seg_chunks) maxc = plan.seg_chunks;
    const int64_t pairs = (int64_t)d->num_seqs * d->heads;
    const int64_t slots = 2 * (int64_t)cus;
    if (pairs > kSplitMaxPairs || maxc < kSplitMinChunks || pairs >= slots) return cut;
    const double step = 3.0, item = 17.0, item_full = 21.2;
    const double items = (double)pairs * (double)maxc;
    // the plain scan: the chain of one pair, the per-chunk stage beside the scan workgroups, or what all scan
    // workgroups together get done (with 64 of them on a busy device a step takes 3.6)
    const double t_scan = (double)maxc * step, t_intra1 = items * item / (double)(slots - pairs);
    const double t_steps = items * (pairs >= 64 ? 3.6 : step) / (double)pairs;
    double best = t_scan > t_intra1 ? t_scan : t_intra1, ratio = 1.0;
    if (t_steps > best) best = t_steps;
    for (int p = 2; p <= split_parts_cap(pairs, plan.seg_chunks); ++p) {
        const int64_t len = (maxc + p - 1) / p;
        if (pairs * (2 * p - 1) * 2 > slots || pairs * p * 8 > slots * 3 || len < 8) continue;
        const bool try_short = len >= kSplitMinTail;
        if (p == 2 && !try_short) continue;                  // two ranges on the general way are the plain scan, later
        int64_t tail = 0;
        const double phase = (double)len * step;
        double t, r = 1.0;
        if (try_short) {
            tail = len / 2 < kSplitMinTail ? kSplitMinTail : len / 2 > kSplitTail ? kSplitTail : len / 2;
            const double t_tails = (double)(p - 1) * (double)tail * (double)pairs * item_full / (double)(slots - pairs * (2 * p - 1));
            const double t_intra = items * item_full / ((double)slots - 0.25 * (double)(pairs * p));
            const double chain = t_tails + (double)tail * step + phase;
            double behind = chain / t_intra - 0.5;
            behind = behind < 0.0 ? 0.0 : behind > 0.5 ? 0.5 : behind;
            const double paced = t_intra * (1.0 + 0.5 * behind);
            t = (chain > paced ? chain : paced) + 0.5 * t_tails;
        } else {
            const double t_intra = items * item / (double)(slots - pairs * (2 * p - 1));
            const double fed = t_intra * (double)(p - 1) / (double)p;
            r = (phase >= 1.5 * fed) ? 0.7 : 1.0;
            t = (phase > fed ? phase : fed) + 60.0 + 12.0 * (p - 2) + phase;
            if (t_intra + 2 * step > t) t = t_intra + 2 * step;
        }
        if (forced >= 2 ? p <= forced : t < best) { best = t; cut.parts = p; ratio = r; cut.tail = tail; }
    }
    if (cut.parts > 1) {
        if (g_split_ratio > 0.0) ratio = g_split_ratio;
        cut.part0_len = (int64_t)((double)plan.seg_chunks * ratio / ((double)(cut.parts - 1) + ratio) + 0.5);
        if (cut.part0_len < 1) cut.part0_len = 1;
        cut.part_len = (plan.seg_chunks - cut.part0_len + cut.parts - 2) / (cut.parts - 1);
        if (g_split_tail >= 0) cut.tail = g_split_tail;
        if (cut.tail > cut.part0_len) cut.tail = cut.part0_len;
        if (cut.tail > cut.part_len) cut.tail = cut.part_len;
    }
    return cut;
}

// The plan with the most chunk indices per segment that fits `workspace_bytes` (full: no limit).
static SegPlan make_plan(const kda_dims *d, size_t workspace_bytes, bool full, bool gate)
{
    const int64_t maxc = max_chunks_per_seq(d);
    int64_t sc = maxc < 1 ? 1 : maxc;
    if (sc > 65535) sc = 65535;                               // a segment holds at most 65 535 chunk indices (4.2 M tokens)
    if (!full) {
        const size_t streams = (size_t)d->num_seqs * d->heads;
        const size_t per_chunk_index = streams * (kSlotBytes + sizeof(uint32_t) + (gate ? kGateSlotBytes : 0));
        const size_t fixed = plan_with(d, 1, gate).total_bytes - per_chunk_index;
        const size_t avail = workspace_bytes > fixed ? workspace_bytes - fixed : 0;
        const int64_t fit = per_chunk_index ? (int64_t)(avail / per_chunk_index) : sc;
        const int64_t most = sc;
        if (fit < sc) sc = fit;
        if (sc < 1) sc = 1;
        // the estimate ignores the rounding of the flag area and the time-split area: settle on the exact sizes
        while (sc > 1 && plan_with(d, sc, gate).total_bytes > workspace_bytes) --sc;
        while (sc < most && plan_with(d, sc + 1, gate).total_bytes <= workspace_bytes) ++sc;
    }
    return plan_with(d, sc, gate);
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

// What a call with this workspace would do: out[0] chunk indices per time segment, [1] time segments,
// [2] ranges of the time-split scan (1: none), [3] length of the first range, [4] of the others (chunks).
kda_status chunk_mfma_plan(const kda_dims *d, size_t workspace_bytes, bool gate, int64_t out[5])
{
    using namespace mfma;
    const SegPlan plan = make_plan(d, workspace_bytes, false, gate);
    if (plan.total_bytes > workspace_bytes) return fail(KDA_ERR_WORKSPACE, "workspace too small for any plan");
    const int cus = compute_units();
    if (cus <= 0) return fail(KDA_ERR_LAUNCH, "cannot query the device");
    const SplitCut cut = g_split ? split_cut(plan, d, cus, g_split) : SplitCut{1, 0, 0, 0};
    out[0] = plan.seg_chunks; out[1] = plan.num_segments; out[2] = cut.parts; out[3] = cut.part0_len; out[4] = cut.part_len;
    return KDA_OK;
}

kda_status chunk_mfma_dispatch(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                               const void *q, const void *k,
                               const void *v, const void *log_alpha, const void *beta, const float *h0,
                               const int32_t *cu, void *o, float *hT, void *workspace,
                               size_t workspace_bytes, bool scalar_gate, hipStream_t stream)
{
    using namespace mfma;
    RawParams raw = {nullptr, nullptr, 0.f};
    if (pro) { raw.a_scale = pro->a_scale; raw.dt_bias = pro->dt_bias; raw.eps = pro->l2norm_eps; }
    const bool out_bf16 = d->out_dtype == KDA_BF16;
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
                hipLaunchKernelGGL(kda_zero_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream,
                                   reinterpret_cast<uint32_t *>(hT), words);
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
    const int cus = compute_units();
    if (cus <= 0) return fail(KDA_ERR_LAUNCH, "cannot query the device");

    uint8_t *base = static_cast<uint8_t *>(workspace);
    uint8_t *ws = base + plan.slots_offset;
    float *carry = hT ? hT : reinterpret_cast<float *>(base + plan.carry_offset);
    uint32_t *flags = reinterpret_cast<uint32_t *>(base + plan.flags_offset);
    uint32_t *status = reinterpret_cast<uint32_t *>(base + plan.status_offset);
    const uint16_t *q16 = static_cast<const uint16_t *>(q), *k16 = static_cast<const uint16_t *>(k),
                   *v16 = static_cast<const uint16_t *>(v), *g16 = static_cast<const uint16_t *>(log_alpha),
                   *b16 = static_cast<const uint16_t *>(beta);
    const int64_t streams = (int64_t)d->num_seqs * d->heads;
    const int64_t maxc = max_chunks_per_seq(d);

    // One launch per time segment, both stages as roles of one kernel.
    const SplitCut cut = g_split ? split_cut(plan, d, cus, g_split) : SplitCut{1, 0, 0, 0};
    const int parts = cut.parts;
    const size_t pair_states = (size_t)streams * D * D;
    for (int64_t seg = 0; seg < plan.num_segments; ++seg) {
        FusedLaunch L{};
        FusedArgs &a = L.args;
        a.q = q16; a.k = k16; a.v = v16; a.log_alpha = g16; a.beta = b16; a.cu = cu;
        a.state_in = (seg == 0) ? h0 : carry;
        a.state_out = (plan.num_segments > 1 || hT) ? carry : nullptr;
        a.o = o; a.ws = ws; a.ready = flags; a.status = status;
        a.T = d->seqlen; a.pairs = streams; a.seg_chunks = plan.seg_chunks; a.seg_index = seg;
        const int64_t left = maxc - seg * plan.seg_chunks;
        a.launch_chunks = left < plan.seg_chunks ? left : plan.seg_chunks;
        a.wait_limit = g_wait_limit; a.H = d->heads; a.scale = d->scale; a.epoch = (uint32_t)(seg + 1);
        a.producers = g_producers; a.raw = raw;
        // packed sequences in more than one batch of pairs: longest first
        const bool ordered = cu != nullptr && parts == 1 && d->num_seqs > 1 && d->num_seqs <= kMaxOrderedSeqs &&
                             streams > fused_batch_pairs(streams, cus);
        a.order = ordered ? reinterpret_cast<const int32_t *>(base + 256) : nullptr;
        L.order_out = (ordered && seg == 0) ? reinterpret_cast<int32_t *>(base + 256) : nullptr;
        L.num_seqs = (int)d->num_seqs;
        a.split.parts = parts; a.split.part_len = cut.part_len; a.split.part0_len = cut.part0_len; a.split.tail = cut.tail;
        a.split.flags = reinterpret_cast<uint32_t *>(base + plan.split_offset);
        a.split.E = reinterpret_cast<float *>(base + plan.split_offset + kSplitFlagBytes);
        a.split.Tm = a.split.E + split_parts_cap((long long)streams, plan.seg_chunks) * pair_states;
        a.split.Bm = a.split.Tm + split_parts_cap((long long)streams, plan.seg_chunks) * pair_states;
        L.raw = pro != nullptr; L.scalar_gate = scalar_gate; L.out_bf16 = out_bf16; L.gate = epi != nullptr;
        if (epi) {
            a.out_gate = static_cast<const uint16_t *>(epi->gate); a.gate_ws = base + plan.gate_offset;
            a.norm_w = epi->norm_weight; a.rms_eps = epi->rms_eps;
        }
        L.reset_flags = seg == 0;
        // (the counters of the time-split scan follow the slot flags: one fill clears both)
        L.num_flags = parts > 1 ? (int64_t)((plan.split_offset + kSplitFlagBytes - plan.flags_offset) / 4)
                                : (int64_t)plan.seg_chunks * streams;
        L.reset_split = parts > 1 && seg > 0;
        L.compute_units = cus;
        const kda_status st = launch_prefill_fused(L, stream);
        if (st != KDA_OK) return st;
    }
    return KDA_OK;
}

}  // namespace kda
