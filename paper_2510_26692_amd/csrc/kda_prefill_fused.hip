// One launch for the whole matrix-core prefill (Section 3.1) of a time segment: the per-chunk
// stage and the sequential stage are two ROLES of one kernel, chosen by workgroup index.
//
// Both roles are workgroups of 256 threads with 80 KiB of LDS, so any two of them share a
// compute unit.  The grid is laid out in batches of `nb` (sequence, head) pairs:
//
//     [ nb scan workgroups ][ nb x chunks per-chunk workgroups, chunk index first ]  [ next batch ] ...
//
// Workgroups are dispatched in index order.  A scan workgroup walks the chunks of its pair and
// takes each slot when the per-chunk workgroup that produces it has raised the slot's flag; the
// per-chunk workgroups wait for nothing.  Every producer a scan workgroup depends on follows it
// in the grid within its own batch, a batch holds at most kMaxBatchPairs scan workgroups, and
// the scan workgroups of the next batch start only when the per-chunk workgroups of this one
// have all been placed: at no time do waiting workgroups hold more than a fraction of the
// device, whatever the number of pairs, so the producers always find room and every wait ends.
// (The wait is bounded anyway: see kda_scan4.h.)
//
// No stream, event or host synchronisation is involved, so the call can be captured into a graph,
// and tools that run one kernel at a time see a single kernel.  The fused output gate of Section 4
// (o <- Sigmoid(g) * RMSNorm(o) * w) is a variant of the same kernel.
#include "kda_prefill_fused.h"

#include "kda_scan4.h"
#include "kda_scan4_split.h"

namespace kda {
namespace mfma {

static_assert(kIntraLds <= scan4::kLds, "both roles run in the LDS of the larger one");
static_assert(kMaxOrderedSeqs == 256, "the fill kernel ranks one sequence per thread of its first workgroup");

// The per-chunk role works through its items (chunk, sequence, head) in the order the scan role wants them,
// per_wg items per workgroup.  `window` consecutive workgroups share a run of window * per_wg items and
// take them in per_wg passes, workgroup r the items r, window + r, 2 window + r, .. of the run: as long as a
// window's workgroups are resident together (the host sizes it for that), the items are finished in nearly the
// order of their index, as they would be with one item per workgroup.
__host__ __device__ inline int64_t intra_workgroups(int64_t items, int per_wg, int window)
{
    const int64_t run = (int64_t)window * per_wg;
    const int64_t full = items / run, rest = items - full * run;
    return full * window + (rest < window ? rest : window);
}
__device__ __forceinline__ int64_t item_index(int64_t wg, int t, int per_wg, int window)
{
    const int64_t w = wg / window, r = wg - w * window;
    return w * window * per_wg + (int64_t)t * window + r;
}
template <bool kGate> __device__ __forceinline__ IntraArgs intra_args(const FusedArgs &a)
{
    return IntraArgs{a.q, a.k, a.v, a.log_alpha, a.beta, a.cu, a.ws, a.T, a.H, a.seg_chunks, a.seg_index, a.scale,
                     a.ready, a.epoch, a.raw, kGate ? a.out_gate : nullptr, kGate ? a.gate_ws : nullptr,
                     kGate ? a.norm_w : nullptr, a.status};
}

// kGate: the output gate of Section 4; the per-chunk role leaves the chunk's gate factors beside its slot and the
// scan role normalises O and applies them in registers (not offered on the scalar-gate entry point).
template <bool kRaw, bool kScalar, bool kOutBf16, bool kGate = false>
__global__ __launch_bounds__(256, 2)
void kda_prefill_kernel(const FusedArgs a)
{
    static_assert(!(kGate && kScalar), "no output gate on the scalar-gate entry point");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (a.split.parts > 1) {
        // ---- time-split layout (few pairs): [pairs x (2 parts - 1) scan workgroups][per-chunk workgroups] ----
        const int nsw = 2 * a.split.parts - 1;
        const int64_t bid = blockIdx.x, nscan = a.pairs * nsw;
        if (bid < nscan) {
            // The workgroups that stay for the length of a range (role 0 and the odd roles) come first, the ones that
            // leave after a tail (the even roles from 2 on) behind them: workgroups are handed to the dies and their
            // shader engines in turn, and role-major order would put all that stay on half of them when there are
            // four or eight pairs (with four pairs, every odd role on dies 4..7).
            const int64_t nstay = a.pairs * a.split.parts;
            const int64_t g = (bid < nstay) ? bid / a.pairs : (bid - nstay) / a.pairs;
            const int64_t pair = (bid < nstay) ? bid - g * a.pairs : bid - nstay - g * a.pairs;
            const int y = (bid < nstay) ? (g == 0 ? 0 : (int)(2 * g - 1)) : (int)(2 * g + 2);
            const int n = (int)(pair / a.H), h = (int)(pair - (int64_t)n * a.H);
            int64_t tok_base, len;
            if (a.cu) { tok_base = a.cu[n]; len = (int64_t)a.cu[n + 1] - tok_base; }
            else      { tok_base = (int64_t)n * a.T; len = a.T; }
            const int64_t cbase = a.seg_index * a.seg_chunks;
            int64_t nchunks = (len + kChunk - 1) / kChunk - cbase;
            if (nchunks < 0) nchunks = 0;
            if (nchunks > a.seg_chunks) nchunks = a.seg_chunks;
            scan4::split_role<kOutBf16, kGate>(lds, a.split, a.ws + pair * a.seg_chunks * (int64_t)kSlotBytes,
                                               a.ready + pair * a.seg_chunks, a.state_in, a.state_out, a.o, pair, a.pairs, y,
                                               tok_base, len, a.H, h, cbase, nchunks, a.epoch, a.status, a.wait_limit,
                                               kGate ? a.gate_ws + pair * a.seg_chunks * (int64_t)kGateSlotBytes : nullptr,
                                               a.rms_eps);
            return;
        }
        if (!a.producers) return;
        // The scan wants the tails of all ranges but the last first (what starts the other ranges comes from
        // them), then walks all ranges side by side: the chunk order is the tails, interleaved, and then the
        // ranges, interleaved, from their starts (a tail's chunks are not produced twice).
        const int64_t parts = a.split.parts, part_len = a.split.part_len, part0_len = a.split.part0_len, tail = a.split.tail;
        const int64_t tails = (parts - 1) * tail;
        const int64_t total = a.pairs * (tails + parts * part_len);
        kda_intra_items<true, kRaw, kScalar>(lds, intra_args<kGate>(a), a.per_wg, [&](int t) __attribute__((always_inline)) {
            const int64_t i = item_index(bid - nscan, t, a.per_wg, a.window);
            IntraItem it = {0, 0, -1};
            if (i >= total) return it;
            const int64_t z = i / a.pairs, pair = i - z * a.pairs;
            int64_t cl;
            if (z < tails) {
                const int64_t rr = z % (parts - 1), j = z / (parts - 1);
                cl = part0_len + rr * part_len - tail + j;                // the end of range rr, less the tail
            } else {
                const int64_t zz = z - tails, rr = zz % parts, j = zz / parts;
                const int64_t rlen = (rr == 0) ? part0_len : part_len;
                if (j >= ((rr == parts - 1) ? rlen : rlen - tail)) return it;
                cl = ((rr == 0) ? 0 : part0_len + (rr - 1) * part_len) + j;
            }
            it.n = (int)(pair / a.H); it.h = (int)(pair - (int64_t)it.n * a.H); it.cl = cl;
            return it;
        });
        return;
    }
    const int64_t batch_items = (int64_t)a.nb * a.launch_chunks;
    const int64_t per_batch = a.nb + intra_workgroups(batch_items, a.per_wg, a.window);
    const int64_t bid = blockIdx.x;
    const int64_t b = bid / per_batch, r = bid - b * per_batch;
    // A batch is a.nb consecutive places; place p is head p % H of the sequence a.order[p / H] (packed calls whose
    // sequences are taken longest first: sequences of like length share a batch, and the batch the grid ends with
    // has the short chains) or of sequence p / H.
    if (r < a.nb) {
        // ---- sequential role: one (sequence, head) ----
        const int64_t place = b * a.nb + r;
        if (place >= a.pairs) return;
        const int64_t seq = place / a.H;
        const int n = a.order ? a.order[seq] : (int)seq, h = (int)(place - seq * a.H);
        const int64_t pair = (int64_t)n * a.H + h;
        int64_t tok_base, len;
        if (a.cu) { tok_base = a.cu[n]; len = (int64_t)a.cu[n + 1] - tok_base; }
        else      { tok_base = (int64_t)n * a.T; len = a.T; }
        const int64_t nchunks = (len + kChunk - 1) / kChunk;
        const int64_t c_begin = a.seg_index * a.seg_chunks;
        const int64_t c_end = (nchunks < c_begin + a.seg_chunks) ? nchunks : c_begin + a.seg_chunks;
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const int64_t st_base = pair * (int64_t)(D * D) + 32 * wave + (lane & 31);
        const uint8_t *slot0 = a.ws + pair * a.seg_chunks * (int64_t)kSlotBytes;
        const scan4::GateParams gate = {kGate ? a.gate_ws + pair * a.seg_chunks * (int64_t)kGateSlotBytes : nullptr, a.rms_eps};
        scan4::kda_scan4_body<true, kOutBf16, kRoleFull, kGate>(lds, slot0, (int64_t)kSlotBytes, a.state_in, a.state_out,
                                                                a.o, st_base, tok_base, len, a.H, c_begin, c_end, h,
                                                                a.ready + pair * a.seg_chunks, a.epoch, a.status,
                                                                a.wait_limit, false, gate);
    } else {
        // ---- per-chunk role: per_wg (chunk, sequence, head) items of this batch, chunk index first ----
        if (!a.producers) return;
        kda_intra_items<true, kRaw, kScalar>(lds, intra_args<kGate>(a), a.per_wg, [&](int t) __attribute__((always_inline)) {
            const int64_t i = item_index(r - a.nb, t, a.per_wg, a.window);
            IntraItem it = {0, 0, -1};
            if (i >= batch_items) return it;
            const int64_t cl = i / a.nb, place = b * a.nb + (i - cl * a.nb);
            if (place >= a.pairs) return it;
            const int64_t seq = place / a.H;
            it.n = a.order ? a.order[seq] : (int)seq; it.h = (int)(place - seq * a.H); it.cl = cl;
            return it;
        });
    }
}

// Clears n words at p and the word at one_more.  Its first workgroup also ranks the sequences of a packed call by
// length when `order` is given: order[rank] = n, longest first (equal lengths: by index), num_seqs <= kMaxOrderedSeqs
// = the 256 threads of the workgroup.
__global__ void kda_fused_fill_kernel(uint32_t *p, int64_t n, uint32_t value, uint32_t *one_more, const int32_t *cu,
                                      int num_seqs, int32_t *order)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
    if (i == 0) *one_more = value;
    if (order == nullptr || blockIdx.x != 0) return;
    __shared__ int32_t len[kMaxOrderedSeqs];
    const int s = threadIdx.x;
    if (s < num_seqs) len[s] = cu[s + 1] - cu[s];
    __syncthreads();
    if (s >= num_seqs) return;
    int rank = 0;
    for (int m = 0; m < num_seqs; ++m) rank += (len[m] > len[s] || (len[m] == len[s] && m < s)) ? 1 : 0;
    order[rank] = s;
}

template <bool kRaw, bool kScalar, bool kOutBf16, bool kGate = false>
static bool reserve_one()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kda_prefill_kernel<kRaw, kScalar, kOutBf16, kGate>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, scan4::kLds) == hipSuccess;
}

static bool reserve_fused_lds()
{
    constexpr int kMaxDevices = 64;
    static bool done[kMaxDevices];                          // same outcome from every thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (done[dev]) return true;
    const bool ok = reserve_one<false, false, false>() && reserve_one<false, false, true>() &&
                    reserve_one<true, false, false>() && reserve_one<true, false, true>() &&
                    reserve_one<false, true, false>() && reserve_one<false, true, true>() &&
                    reserve_one<false, false, false, true>() && reserve_one<false, false, true, true>() &&
                    reserve_one<true, false, false, true>() && reserve_one<true, false, true, true>();
    if (!ok) (void)hipGetLastError();
    done[dev] = ok;
    return ok;
}

int fused_batch_pairs(int64_t pairs, int compute_units)
{
    int most = compute_units / 2;                             // a quarter of the two slots per compute unit
    if (most > kMaxBatchPairs) most = kMaxBatchPairs;
    if (most < 1) most = 1;
    return (int)(pairs < most ? pairs : most);
}

kda_status launch_prefill_fused(const FusedLaunch &L, hipStream_t stream)
{
    if (!reserve_fused_lds())
        return fail(KDA_ERR_LAUNCH, "cannot reserve %d bytes of LDS for the prefill kernel", scan4::kLds);
    FusedArgs a = L.args;
    a.nb = fused_batch_pairs(a.pairs, L.compute_units);
    int64_t blocks;
    // chunks per workgroup of the per-chunk role, and the workgroups of that role expected to be resident
    // together: two per compute unit, less the scan workgroups beside them (two batches' worth, or all of them)
    const int slots = 2 * L.compute_units;
    a.per_wg = kItemsPerWorkgroup;
    if (a.split.parts > 1) {
        const int64_t nscan = a.pairs * (int64_t)(2 * a.split.parts - 1);
        a.window = (int)(slots - nscan > 64 ? slots - nscan : 64);
        const int64_t items = a.pairs * ((a.split.parts - 1) * a.split.tail + (int64_t)a.split.parts * a.split.part_len);
        blocks = nscan + intra_workgroups(items, a.per_wg, a.window);
    } else {
        const int64_t nbatches = (a.pairs + a.nb - 1) / a.nb;
        const int64_t beside = nbatches > 1 ? 2 * a.nb : a.nb;
        a.window = (int)(slots - beside > 64 ? slots - beside : 64);
        blocks = nbatches * (a.nb + intra_workgroups((int64_t)a.nb * a.launch_chunks, a.per_wg, a.window));
    }
    if (blocks > 0x7fffffffLL)
        return fail(KDA_ERR_UNSUPPORTED, "%lld workgroups in one launch: use a smaller workspace (shorter time segments)",
                    (long long)blocks);
    if (L.reset_split)
        hipLaunchKernelGGL(kda_fused_fill_kernel, dim3((unsigned)(kSplitFlagBytes / 4 / 256)), dim3(256), 0, stream,
                           a.split.flags, (int64_t)(kSplitFlagBytes / 4), 0u, a.split.flags, nullptr, 0, nullptr);
    // the slot flags and the status word start every call at zero (a kernel, not a memset: the call may be captured)
    if (L.reset_flags)
        hipLaunchKernelGGL(kda_fused_fill_kernel, dim3((unsigned)((L.num_flags + 255) / 256 + 1)), dim3(256), 0, stream,
                           a.ready, L.num_flags, 0u, a.status, a.cu, L.num_seqs, L.order_out);
    if (L.gate && L.scalar_gate)
        return fail(KDA_ERR_UNSUPPORTED, "the scalar-gate entry point has no output gate");
    auto kern = L.gate ? (L.raw ? (L.out_bf16 ? kda_prefill_kernel<true, false, true, true> : kda_prefill_kernel<true, false, false, true>)
                                : (L.out_bf16 ? kda_prefill_kernel<false, false, true, true> : kda_prefill_kernel<false, false, false, true>))
                : L.scalar_gate ? (L.out_bf16 ? kda_prefill_kernel<false, true, true> : kda_prefill_kernel<false, true, false>)
                : L.raw ? (L.out_bf16 ? kda_prefill_kernel<true, false, true> : kda_prefill_kernel<true, false, false>)
                        : (L.out_bf16 ? kda_prefill_kernel<false, false, true> : kda_prefill_kernel<false, false, false>);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), scan4::kLds, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_prefill_kernel: %s", hipGetErrorString(e));
    return KDA_OK;
}

}  // namespace mfma
}  // namespace kda

#ifdef KDA_SCAN4_TRACE
extern "C" int kda_debug_read_trace(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(kda::mfma::scan4::g_trace), sizeof(unsigned long long) * 64 * 8, 0, hipMemcpyDeviceToHost);
}
#endif
