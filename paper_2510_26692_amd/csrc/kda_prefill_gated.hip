// The matrix-core prefill with the fused output gate of Section 4 (o <- Sigmoid(g) * RMSNorm(o) * w):
// two kernels per time segment on the caller's stream, one after the other.
//
//  kda_intra_gate   one workgroup per (chunk, head): the per-chunk stage (kda_intra.h), which also
//                   re-lays the chunk's gate logits into the accumulator order of the scan.
//  kda_scan_gate    one workgroup of eight waves per (sequence, head): the sequential stage with the
//                   gate applied to O in registers before the store (kda_scan8.h).
//
// Every other call takes the one-kernel path of kda_prefill_fused.hip.
#include "kda_prefill_gated.h"

#include "kda_scan8.h"

namespace kda {
namespace mfma {

template <bool kRaw>
__global__ __launch_bounds__(256, 2)
void kda_intra_gate_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
                           const uint16_t *__restrict__ v, const uint16_t *__restrict__ log_alpha,
                           const uint16_t *__restrict__ beta, const int32_t *__restrict__ cu_seqlens,
                           uint8_t *__restrict__ ws, int64_t T, int H, int64_t seg_chunks, int64_t seg_index,
                           float scale, RawParams raw, const uint16_t *__restrict__ out_gate,
                           uint8_t *__restrict__ gate_ws)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // x = head, y = chunk, z = sequence: consecutive workgroups read neighbouring tokens
    const IntraArgs A = {q, k, v, log_alpha, beta, cu_seqlens, ws, T, H, seg_chunks, seg_index, scale, nullptr, 0u, raw,
                         out_gate, gate_ws, nullptr};
    kda_intra_items<false, kRaw, false>(lds, A, 1, [&](int) __attribute__((always_inline)) {
        return IntraItem{(int)blockIdx.x, (int)blockIdx.z, (int64_t)blockIdx.y};
    });
}

static bool reserve_gated_lds()
{
    constexpr int kMaxDevices = 64;
    static bool done[kMaxDevices];                          // same outcome from every thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (done[dev]) return true;
    const bool ok =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_gate_kernel<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_intra_gate_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kIntraLds) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(kda_scan_kernel<false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, scan::kLds) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    done[dev] = ok;
    return ok;
}

kda_status launch_prefill_gated(const GatedLaunch &L, hipStream_t stream)
{
    if (!reserve_gated_lds())
        return fail(KDA_ERR_LAUNCH, "cannot reserve LDS for the gated prefill kernels (%d, %d bytes)", kIntraLds,
                    (int)scan::kLds);
    EpiParams ep = {L.gate, L.norm_w, L.rms_eps, L.out_bf16 ? 1 : 0, L.gate_ws};
    const dim3 grid((unsigned)L.H, (unsigned)L.launch_chunks, (unsigned)L.num_seqs);
    auto intra = L.raw_inputs ? kda_intra_gate_kernel<true> : kda_intra_gate_kernel<false>;
    hipLaunchKernelGGL(intra, grid, dim3(256), kIntraLds, stream, L.q, L.k, L.v, L.log_alpha, L.beta, L.cu, L.ws, L.T, L.H,
                       L.seg_chunks, L.seg_index, L.scale, L.raw, L.gate, L.gate_ws);
    hipLaunchKernelGGL((kda_scan_kernel<false, true>), dim3((unsigned)((int64_t)L.num_seqs * L.H)), dim3(512), scan::kLds, stream,
                       L.ws, L.state_in, L.state_out, L.cu, L.o, L.T, L.H, L.seg_chunks, L.seg_index,
                       (const uint32_t *)nullptr, 0u, L.status, ep);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "gated prefill kernels: %s", hipGetErrorString(e));
    return KDA_OK;
}

}  // namespace mfma
}  // namespace kda
