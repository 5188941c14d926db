// Diagnostic probes (kda_debug.h): the device's own streaming and matrix-core rates, measured with the
// simplest kernels that reach them, so that a roofline fraction of a KDA kernel can be read against
// what this device delivers as well as against its data-sheet peaks.
#include "kda_common.h"
#include "kda_debug.h"

namespace kda {

constexpr int kProbeTile = 16384;            // floats per workgroup: 64 KiB, one decode state

// mode 0: read only, 1: write only, 2: read, modify and write in place (the decode step's traffic)
template <int kMode>
__global__ __launch_bounds__(256) void kda_stream_probe_kernel(float *buf, float a)
{
    f32x4 *p = reinterpret_cast<f32x4 *>(buf + (size_t)blockIdx.x * kProbeTile) + threadIdx.x;
    f32x4 s[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        if (kMode == 1) { const f32x4 c = {a, a, a, a}; s[m] = c; }
        else            s[m] = __builtin_nontemporal_load(p + m * 256);
    }
    float acc = 0.f;
#pragma unroll
    for (int m = 0; m < 16; ++m) { s[m] = s[m] * a + 1.0f; acc += s[m][0]; }
    if (kMode != 0) {
#pragma unroll
        for (int m = 0; m < 16; ++m) __builtin_nontemporal_store(s[m], p + m * 256);
    } else if (acc == 12345.678f) {
        p[0] = s[0];                          // (never taken: keeps the loads alive)
    }
}

// mode 3: the data movement of the two-stage prefill and nothing else.  Item i (one chunk of one head) reads 64 KiB of
// streamed input, writes a 72 KiB slot, reads the slot of another item (written by another workgroup) and writes
// 32 KiB of streamed output: 240 KiB through the memory system per item, as kda_prefill_kernel moves per chunk with
// bf16 inputs and fp32 o.  The buffer holds `items` records of 168 KiB: [64 KiB in][72 KiB slot][32 KiB out].
constexpr int kItemIn = 65536, kItemSlot = 73728, kItemOut = 32768, kItemBytes = kItemIn + kItemSlot + kItemOut;
__global__ __launch_bounds__(256) void kda_prefill_traffic_probe_kernel(uint8_t *buf, unsigned items, float a)
{
    const unsigned i = blockIdx.x, j = (i + items / 2) % items;
    const f32x4 *in = reinterpret_cast<const f32x4 *>(buf + (size_t)i * kItemBytes) + threadIdx.x;
    f32x4 *slot = reinterpret_cast<f32x4 *>(buf + (size_t)i * kItemBytes + kItemIn) + threadIdx.x;
    const f32x4 *other = reinterpret_cast<const f32x4 *>(buf + (size_t)j * kItemBytes + kItemIn) + threadIdx.x;
    f32x4 *out = reinterpret_cast<f32x4 *>(buf + (size_t)i * kItemBytes + kItemIn + kItemSlot) + threadIdx.x;
    f32x4 acc = {a, a, a, a};
#pragma unroll
    for (int m = 0; m < kItemIn / 4096; ++m) acc += __builtin_nontemporal_load(in + m * 256);
#pragma unroll
    for (int m = 0; m < kItemSlot / 4096; ++m) __builtin_nontemporal_store(acc, slot + m * 256);
#pragma unroll
    for (int m = 0; m < kItemSlot / 4096; ++m) acc += __builtin_nontemporal_load(other + m * 256);
#pragma unroll
    for (int m = 0; m < kItemOut / 4096; ++m) __builtin_nontemporal_store(acc, out + m * 256);
}

// Every wave issues 16 * iters products 32x32x16 (f16 in, fp32 out) on four independent accumulators.
__global__ __launch_bounds__(256) void kda_mfma_probe_kernel(float *sink, int iters)
{
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    const _Float16 x = (_Float16)(1.0f + (float)(threadIdx.x & 7) * 0.125f);
    const h8 a = {x, x, x, x, x, x, x, x}, b = {x, -x, x, -x, x, -x, x, -x};
    f32x16 c0 = {0.f}, c1 = {0.f}, c2 = {0.f}, c3 = {0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
        }
    }
    const f32x16 c = c0 + c1 + c2 + c3;
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) t += c[j];
    if (t == 12345.678f) sink[0] = t;         // (never taken: keeps the products alive)
}

}  // namespace kda

using namespace kda;

extern "C" kda_status kda_debug_stream_probe(int mode, float *buffer, size_t bytes, void *hip_stream)
{
    if (mode < 0 || mode > 2) return fail(KDA_ERR_INVALID_ARG, "mode must be 0, 1 or 2, got %d", mode);
    if (!buffer || bytes == 0 || bytes % (kProbeTile * sizeof(float)) != 0 || (reinterpret_cast<uintptr_t>(buffer) & 15u))
        return fail(KDA_ERR_INVALID_ARG, "buffer must be 16-byte aligned and a multiple of 65536 bytes long");
    const size_t blocks = bytes / (kProbeTile * sizeof(float));
    if (blocks > 0x7fffffffu) return fail(KDA_ERR_INVALID_ARG, "buffer too large");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    auto kern = mode == 0 ? kda_stream_probe_kernel<0> : mode == 1 ? kda_stream_probe_kernel<1> : kda_stream_probe_kernel<2>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, stream, buffer, 0.5f);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_stream_probe_kernel: %s", hipGetErrorString(e));
    return KDA_OK;
}

extern "C" kda_status kda_debug_prefill_traffic_probe(void *buffer, size_t bytes, size_t *moved, void *hip_stream)
{
    if (!buffer || bytes < 2 * (size_t)kItemBytes || bytes % kItemBytes != 0 || (reinterpret_cast<uintptr_t>(buffer) & 15u))
        return fail(KDA_ERR_INVALID_ARG, "buffer must be 16-byte aligned and a multiple (at least two) of %d bytes long", kItemBytes);
    const size_t items = bytes / kItemBytes;
    if (items > 0x7fffffffu) return fail(KDA_ERR_INVALID_ARG, "buffer too large");
    hipLaunchKernelGGL(kda_prefill_traffic_probe_kernel, dim3((unsigned)items), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<uint8_t *>(buffer), (unsigned)items, 0.5f);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_prefill_traffic_probe_kernel: %s", hipGetErrorString(e));
    if (moved) *moved = items * (size_t)(kItemIn + 2 * kItemSlot + kItemOut);
    return KDA_OK;
}

extern "C" kda_status kda_debug_mfma_probe(float *sink, int workgroups, int iters, double *flops, void *hip_stream)
{
    if (!sink || workgroups <= 0 || iters <= 0) return fail(KDA_ERR_INVALID_ARG, "sink, workgroups and iters must be given");
    hipLaunchKernelGGL(kda_mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream), sink, iters);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_mfma_probe_kernel: %s", hipGetErrorString(e));
    if (flops) *flops = (double)workgroups * 4.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
    return KDA_OK;
}
