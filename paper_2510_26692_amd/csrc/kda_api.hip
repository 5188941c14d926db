// C ABI of libkda: argument validation, error strings and dispatch to the
// kernels.  Nothing here touches tensor data; every step of the path runs in
// the kernels of kda_step.hip, kda_chunk_f32.hip, kda_prefill_fused.hip and kda_chunk_bwd.hip.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kda_common.h"
#include "kda_debug.h"

namespace kda {

static thread_local char g_last_error[512] = "";

kda_status fail(kda_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
    return code;
}

// Kernel-side entry points (one per source file).
kda_status recurrent_step_dispatch(const kda_dims *, const kda_prologue *, const kda_epilogue *, const void *, const void *,
                                   const void *, const void *, const void *, float *, void *,
                                   const int32_t *, bool scalar_gate, hipStream_t);
int recurrent_max_steps();
kda_status chunk_f32_dispatch(const kda_dims *, const void *, const void *, const void *,
                              const void *, const void *, const float *, const int32_t *, void *,
                              float *, hipStream_t);
kda_status chunk_mfma_dispatch(const kda_dims *, const kda_prologue *, const kda_epilogue *, const void *, const void *, const void *,
                               const void *, const void *, const float *, const int32_t *, void *,
                               float *, void *, size_t, bool scalar_gate, hipStream_t);
size_t chunk_mfma_workspace_size(const kda_dims *, bool minimal, bool output_gate);
size_t chunk_mfma_status_offset(const kda_dims *, size_t workspace_bytes);
kda_status chunk_mfma_plan(const kda_dims *, size_t workspace_bytes, bool gate, int64_t out[5]);
size_t chunk_bwd_workspace_size(const kda_dims *);
size_t chunk_f32_fast_workspace_size(const kda_dims *);
kda_status chunk_f32_fast_dispatch(const kda_dims *, const void *, const void *, const void *, const void *,
                                   const void *, const float *, const int32_t *, void *, float *, void *,
                                   hipStream_t);
kda_status chunk_bwd_dispatch(const kda_dims *, const void *, const void *, const void *, const void *,
                              const void *, const float *, const int32_t *, const void *, const float *,
                              float *, float *, float *, float *, float *, float *, void *, size_t,
                              hipStream_t);

// Diagnostics switches (kda_debug.h): process-wide, read at the start of a call.
// 0 keeps the sequential stage of the matrix-core prefill to one workgroup per (sequence, head) whatever
// the shape (kda_debug_set_time_split, or KDA_PREFILL_TIME_SPLIT=0 in the environment).
static int split_default()
{
    const char *e = getenv("KDA_PREFILL_TIME_SPLIT");
    return (e && e[0] == '0' && e[1] == 0) ? 0 : 1;
}
int g_split = split_default();
// development switch: length of the first range of the time-split scan relative to the others
// (0 = chosen per call)
static double split_ratio_default()
{
    const char *e = getenv("KDA_PREFILL_SPLIT_RATIO");
    const double r = e ? atof(e) : 0.0;
    return (r >= 0.2 && r <= 1.0) ? r : 0.0;
}
double g_split_ratio = split_ratio_default();
// development switch: chunks at a range's end that the time-split scan tests for a vanished transition
// (-1 = chosen per call, 0 = not tried)
static int split_tail_default()
{
    const char *e = getenv("KDA_PREFILL_SPLIT_TAIL");
    const int t = e ? atoi(e) : -1;
    return (e && t >= 0 && t <= 4096) ? t : -1;
}
int g_split_tail = split_tail_default();
int g_producers = 1;                      // 0: the per-chunk role of the one-kernel prefill does nothing
uint64_t g_wait_limit = 200000000ull;     // ticks of the 100 MHz wall clock a scan workgroup waits for a slot: two seconds

// Scratch of the entry point that allocates nothing (kda_chunk_fwd_static_scratch): each device the
// library runs on holds its own copy of this array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (the array's name is a host-side stand-in, not a
// device address): asked once per device, with that device current, and kept.
static kda_status static_scratch_ptr(void **out)
{
    constexpr int kMaxDevices = 64;
    static void *table[kMaxDevices];                        // same value from every thread
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return fail(KDA_ERR_LAUNCH, "cannot tell the current device");
    }
    if (!table[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return fail(KDA_ERR_LAUNCH, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        }
        table[dev] = ptr;
    }
    *out = table[dev];
    return KDA_OK;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by both entry points.  Returns KDA_OK or the failure code.
static kda_status check_dims(const kda_dims *d, bool packed)
{
    if (!d) return fail(KDA_ERR_INVALID_ARG, "dims is NULL");
    if (d->batch < 0 || d->seqlen < 0 || d->heads < 0 || d->num_seqs < 0)
        return fail(KDA_ERR_INVALID_ARG, "negative size (batch %d, seqlen %lld, heads %d, num_seqs %d)",
                    d->batch, (long long)d->seqlen, d->heads, d->num_seqs);
    if (d->in_dtype != KDA_F32 && d->in_dtype != KDA_BF16)
        return fail(KDA_ERR_INVALID_ARG, "in_dtype %d is not a kda_dtype", (int)d->in_dtype);
    if (d->out_dtype != KDA_F32 && d->out_dtype != KDA_BF16)
        return fail(KDA_ERR_INVALID_ARG, "out_dtype %d is not a kda_dtype", (int)d->out_dtype);
    if (d->out_dtype == KDA_BF16 && d->in_dtype != KDA_BF16)
        return fail(KDA_ERR_UNSUPPORTED, "out_dtype KDA_BF16 needs in_dtype KDA_BF16");
    if (!(d->dk == d->dv && (d->dk == 64 || d->dk == 128)))
        return fail(KDA_ERR_UNSUPPORTED, "head dims must satisfy dk == dv in {64,128}, got %d x %d",
                    d->dk, d->dv);
    if (d->heads > 65535) return fail(KDA_ERR_UNSUPPORTED, "heads > 65535");
    if (packed) {
        if (d->batch != 1) return fail(KDA_ERR_INVALID_ARG, "packed batches need batch == 1");
        if (d->seqlen > 0x7fffffffLL)
            return fail(KDA_ERR_INVALID_ARG, "packed token count exceeds the int32 range of cu_seqlens");
        if (d->max_seqlen < 0) return fail(KDA_ERR_INVALID_ARG, "max_seqlen < 0");
    } else if (d->num_seqs != d->batch) {
        return fail(KDA_ERR_INVALID_ARG, "fixed-length batches need num_seqs == batch");
    }
    if (!(d->scale == d->scale)) return fail(KDA_ERR_INVALID_ARG, "scale is NaN");
    return KDA_OK;
}

static bool mfma_path(const kda_dims *d)
{
    if (d->in_dtype != KDA_BF16) return false;
    if (d->dk != 128) return false;                     // bf16 inputs with head dim 64 take the fp32 kernels
    const char *force = getenv("KDA_CHUNK_IMPL");       // debugging switch: "f32" forces the
    if (force && strcmp(force, "f32") == 0) return false;  // fp32 kernel for bf16 inputs too
    return true;
}

}  // namespace kda

using namespace kda;

extern "C" {

const char *kda_version(void) { return "kda-gfx950 0.1"; }

void kda_debug_set_producers(int enabled) { g_producers = enabled ? 1 : 0; }

void kda_debug_set_wait_limit(unsigned long long ticks) { g_wait_limit = ticks; }

void kda_debug_set_time_split(int mode) { g_split = mode < 0 ? 0 : mode; }

kda_status kda_debug_chunk_fwd_plan(const kda_dims *d, size_t workspace_bytes, int output_gate, int64_t out[5])
{
    g_last_error[0] = 0;
    if (!d || !out) return fail(KDA_ERR_INVALID_ARG, "dims or out is NULL");
    if (d->chunk != kChunk) return fail(KDA_ERR_UNSUPPORTED, "chunk must be %d, got %d", kChunk, d->chunk);
    const kda_status st = check_dims(d, d->num_seqs != d->batch);
    if (st != KDA_OK) return st;
    if (!mfma_path(d)) return fail(KDA_ERR_UNSUPPORTED, "only the matrix-core prefill (bf16 inputs, dk = dv = 128) has a plan");
    if (d->seqlen == 0 || d->num_seqs == 0 || d->heads == 0) { out[0] = out[1] = out[3] = out[4] = 0; out[2] = 1; return KDA_OK; }
    return chunk_mfma_plan(d, workspace_bytes, output_gate != 0, out);
}

const char *kda_last_error(void) { return g_last_error; }

const char *kda_status_string(kda_status s)
{
    switch (s) {
    case KDA_OK: return "ok";
    case KDA_ERR_INVALID_ARG: return "invalid argument";
    case KDA_ERR_UNSUPPORTED: return "unsupported configuration";
    case KDA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KDA_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

static size_t workspace_size(const kda_dims *d, bool minimal, bool output_gate)
{
    if (!d || d->chunk != kChunk) return 0;
    const char saved0 = g_last_error[0];
    if (check_dims(d, d->num_seqs != d->batch) != KDA_OK) { g_last_error[0] = saved0; return 0; }
    // the fp32 path runs without a workspace (one sequential kernel) and much faster with one
    if (!mfma_path(d)) return (minimal || d->seqlen == 0) ? 0 : chunk_f32_fast_workspace_size(d);
    return chunk_mfma_workspace_size(d, minimal, output_gate);
}

size_t kda_chunk_fwd_workspace_size(const kda_dims *d) { return workspace_size(d, false, false); }
size_t kda_chunk_fwd_min_workspace_size(const kda_dims *d) { return workspace_size(d, true, false); }
size_t kda_chunk_fwd_fused_workspace_size(const kda_dims *d, const kda_epilogue *epi)
{
    return workspace_size(d, false, epi != nullptr);
}
size_t kda_chunk_fwd_fused_min_workspace_size(const kda_dims *d, const kda_epilogue *epi)
{
    return workspace_size(d, true, epi != nullptr);
}

size_t kda_chunk_bwd_workspace_size(const kda_dims *d)
{
    if (!d || d->chunk != kChunk) return 0;
    const char saved0 = g_last_error[0];
    if (check_dims(d, d->num_seqs != d->batch) != KDA_OK) { g_last_error[0] = saved0; return 0; }
    return chunk_bwd_workspace_size(d);
}

kda_status kda_chunk_bwd(const kda_dims *d, const void *q, const void *k, const void *v,
                         const void *log_alpha, const void *beta, const float *h0,
                         const int32_t *cu_seqlens, const void *d_o, const float *d_hT,
                         float *dq, float *dk, float *dv, float *dlog_alpha, float *dbeta, float *dh0,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    kda_status st = check_dims(d, cu_seqlens != nullptr);
    if (st != KDA_OK) return st;
    if (d->chunk != kChunk) return fail(KDA_ERR_UNSUPPORTED, "chunk must be %d, got %d", kChunk, d->chunk);
    const bool empty = d->seqlen == 0 || d->heads == 0 || d->batch == 0;
    if (!empty && (!q || !k || !v || !log_alpha || !beta || !d_o || !dq || !dk || !dv || !dlog_alpha || !dbeta))
        return fail(KDA_ERR_INVALID_ARG, "inputs, d_o and the five per-token gradients must be non-NULL");
    const void *ptrs[] = {q, k, v, log_alpha, beta, h0, d_o, d_hT, dq, dk, dv, dlog_alpha, dbeta, dh0};
    for (const void *p : ptrs)
        if (!aligned16(p)) return fail(KDA_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u)
        return fail(KDA_ERR_INVALID_ARG, "cu_seqlens must be 4-byte aligned");
    if (reinterpret_cast<uintptr_t>(workspace) & 255u)
        return fail(KDA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (!empty) {
        const void *outs[] = {dq, dk, dv, dlog_alpha, dbeta, dh0};
        const void *ins[] = {q, k, v, log_alpha, beta, h0, d_o, d_hT};
        for (int a = 0; a < 6; ++a) {
            if (!outs[a]) continue;
            for (const void *in : ins)
                if (outs[a] == in) return fail(KDA_ERR_INVALID_ARG, "a gradient must not alias an input");
            for (int b = a + 1; b < 6; ++b)
                if (outs[a] == outs[b]) return fail(KDA_ERR_INVALID_ARG, "gradients must not alias each other");
        }
    }
    if (d->num_seqs == 0 || d->heads == 0) return KDA_OK;
    if (d->seqlen == 0 && !dh0) return KDA_OK;            // no tokens and nobody asks for dh0 = d_hT
    return chunk_bwd_dispatch(d, q, k, v, log_alpha, beta, h0, cu_seqlens, d_o, d_hT, dq, dk, dv, dlog_alpha,
                              dbeta, dh0, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

static kda_status check_epilogue(const kda_epilogue *epi)
{
    if (!epi) return KDA_OK;
    if (!(epi->rms_eps >= 0.f)) return fail(KDA_ERR_INVALID_ARG, "rms_eps must be >= 0");
    if (!epi->gate || !aligned16(epi->gate) || (reinterpret_cast<uintptr_t>(epi->norm_weight) & 15u))
        return fail(KDA_ERR_INVALID_ARG, "epilogue gate must be non-NULL; gate and norm_weight 16-byte aligned");
    return KDA_OK;
}

static kda_status check_prologue(const kda_prologue *pro)
{
    if (!pro) return KDA_OK;
    if (!(pro->l2norm_eps >= 0.f)) return fail(KDA_ERR_INVALID_ARG, "l2norm_eps must be >= 0");
    if ((reinterpret_cast<uintptr_t>(pro->a_scale) & 3u) || (reinterpret_cast<uintptr_t>(pro->dt_bias) & 3u))
        return fail(KDA_ERR_INVALID_ARG, "a_scale and dt_bias must be 4-byte aligned");
    return KDA_OK;
}

static kda_status chunk_fwd_impl(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                                 const void *q, const void *k,
                                 const void *v, const void *log_alpha, const void *beta, const float *h0,
                                 const int32_t *cu_seqlens, void *o, float *hT, void *workspace,
                                 size_t workspace_bytes, void *hip_stream, bool scalar_gate = false)
{
    kda_status st = check_dims(d, cu_seqlens != nullptr);
    if (st != KDA_OK) return st;
    if (scalar_gate && !(d->in_dtype == KDA_BF16 && d->dk == 128 && d->dv == 128 && mfma_path(d)))
        return fail(KDA_ERR_UNSUPPORTED, "the scalar-gate prefill is built for bf16 inputs with dk == dv == 128");
    if ((pro || epi) && !(d->in_dtype == KDA_BF16 && d->dk == 128 && d->dv == 128))
        return fail(KDA_ERR_UNSUPPORTED, "the fused stages are built for bf16 inputs with dk == dv == 128");
    if (epi && (o == epi->gate)) return fail(KDA_ERR_INVALID_ARG, "o must not alias the output gate");
    if (d->chunk != kChunk) return fail(KDA_ERR_UNSUPPORTED, "chunk must be %d, got %d", kChunk, d->chunk);
    const bool empty = d->seqlen == 0 || d->heads == 0 || d->batch == 0;
    if (!empty && (!q || !k || !v || !log_alpha || !beta || !o))
        return fail(KDA_ERR_INVALID_ARG, "q, k, v, log_alpha, beta and o must be non-NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(log_alpha) || !aligned16(beta) ||
        !aligned16(o) || !aligned16(h0) || !aligned16(hT) || (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u))
        return fail(KDA_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (o == q || o == k || o == v || o == log_alpha || o == beta)
        if (!empty) return fail(KDA_ERR_INVALID_ARG, "o must not alias an input");
    if (d->num_seqs == 0 || d->heads == 0) return KDA_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    if (!mfma_path(d)) {
        if (pro || epi) return fail(KDA_ERR_UNSUPPORTED, "the fused stages need the matrix-core prefill");
        if (d->out_dtype != KDA_F32) return fail(KDA_ERR_UNSUPPORTED, "the fp32 prefill kernels write fp32 outputs only");
        const size_t fast = d->seqlen == 0 ? 0 : chunk_f32_fast_workspace_size(d);
        if (fast > 0 && workspace && workspace_bytes >= fast && !(reinterpret_cast<uintptr_t>(workspace) & 255u))
            return chunk_f32_fast_dispatch(d, q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, workspace, stream);
        return chunk_f32_dispatch(d, q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, stream);
    }

    const size_t need = chunk_mfma_workspace_size(d, true, epi != nullptr);
    if (need > 0) {
        if (!workspace) return fail(KDA_ERR_WORKSPACE, "workspace is NULL, at least %zu bytes needed", need);
        if (reinterpret_cast<uintptr_t>(workspace) & 255u)
            return fail(KDA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
        if (workspace_bytes < need)
            return fail(KDA_ERR_WORKSPACE, "workspace has %zu bytes, at least %zu needed", workspace_bytes, need);
    }
    return chunk_mfma_dispatch(d, pro, epi, q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, workspace,
                               workspace_bytes, scalar_gate, stream);
}

kda_status kda_chunk_fwd(const kda_dims *d, const void *q, const void *k, const void *v,
                         const void *log_alpha, const void *beta, const float *h0,
                         const int32_t *cu_seqlens, void *o, float *hT, void *workspace,
                         size_t workspace_bytes, void *hip_stream)
{
    g_last_error[0] = 0;
    return chunk_fwd_impl(d, nullptr, nullptr, q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, workspace,
                          workspace_bytes, hip_stream);
}

size_t kda_static_scratch_size(void) { return kStaticScratchBytes; }

kda_status kda_chunk_fwd_static_scratch(const kda_dims *d, const void *q, const void *k, const void *v,
                                        const void *log_alpha, const void *beta, const float *h0,
                                        const int32_t *cu_seqlens, void *o, float *hT, void *hip_stream)
{
    g_last_error[0] = 0;
    kda_status st = check_dims(d, cu_seqlens != nullptr);
    if (st != KDA_OK) return st;
    if (d->chunk != kChunk) return fail(KDA_ERR_UNSUPPORTED, "chunk must be %d, got %d", kChunk, d->chunk);
    // the smallest workspace the call can run with must fit the array (KDA_F32 inputs need none at all)
    const size_t need = mfma_path(d) ? chunk_mfma_workspace_size(d, true, false) : 0;
    if (need > kStaticScratchBytes)
        return fail(KDA_ERR_WORKSPACE, "this call needs at least %zu bytes of scratch, the static array holds %zu: fewer "
                    "sequences or heads per call", need, kStaticScratchBytes);
    void *ptr = nullptr;
    st = static_scratch_ptr(&ptr);
    if (st != KDA_OK) return st;
    return chunk_fwd_impl(d, nullptr, nullptr, q, k, v, log_alpha, beta, h0, cu_seqlens, o, hT, ptr, kStaticScratchBytes,
                          hip_stream);
}

kda_status kda_chunk_fwd_scalar_gate(const kda_dims *d, const void *q, const void *k, const void *v,
                                     const void *log_alpha_head, const void *beta, const float *h0,
                                     const int32_t *cu_seqlens, void *o, float *hT, void *workspace,
                                     size_t workspace_bytes, void *hip_stream)
{
    g_last_error[0] = 0;
    return chunk_fwd_impl(d, nullptr, nullptr, q, k, v, log_alpha_head, beta, h0, cu_seqlens, o, hT, workspace,
                          workspace_bytes, hip_stream, true);
}

kda_status kda_chunk_fwd_fused(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                               const void *q_raw, const void *k_raw, const void *v, const void *gate, const void *beta_logit,
                               const float *h0, const int32_t *cu_seqlens, void *o, float *hT,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    g_last_error[0] = 0;
    kda_status st = check_prologue(pro);
    if (st == KDA_OK) st = check_epilogue(epi);
    if (st != KDA_OK) return st;
    return chunk_fwd_impl(d, pro, epi, q_raw, k_raw, v, gate, beta_logit, h0, cu_seqlens, o, hT, workspace,
                          workspace_bytes, hip_stream);
}

kda_status kda_chunk_fwd_check(const kda_dims *d, const void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    g_last_error[0] = 0;
    if (!d) return fail(KDA_ERR_INVALID_ARG, "dims is NULL");
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "stream: %s", hipGetErrorString(e));
    if (d->chunk != kChunk || check_dims(d, d->num_seqs != d->batch) != KDA_OK) return KDA_ERR_INVALID_ARG;
    if (!mfma_path(d) || !workspace || chunk_mfma_workspace_size(d, true, false) == 0 ||
        workspace_bytes < chunk_mfma_workspace_size(d, true, false))
        return KDA_OK;                                       // this path leaves no status word
    uint32_t word = 0;
    e = hipMemcpy(&word, static_cast<const uint8_t *>(workspace) + chunk_mfma_status_offset(d, workspace_bytes),
                  sizeof(word), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "status read: %s", hipGetErrorString(e));
    if (word & 1u)
        return fail(KDA_ERR_LAUNCH, "the sequential stage gave up waiting for a workspace slot (status %u): o is NaN from "
                    "that point of each affected (sequence, head) on, and so is a final state computed from there", word);
    if (word & 4u)
        return fail(KDA_ERR_INVALID_ARG, "a key outside the domain of the fp16 matrix-core operands (status %u): |k_t|^2 > 16 "
                    "for some token; the results may be inaccurate or not finite", word);
    if (word & 2u)
        return fail(KDA_ERR_INVALID_ARG, "a state left the range of the fp16 matrix-core operands (status %u): inputs outside "
                    "the documented domain; the affected outputs are Inf or NaN", word);
    return KDA_OK;
}

kda_status kda_debug_chunk_fwd_status(const kda_dims *d, const void *workspace, size_t workspace_bytes,
                                      void *hip_stream, unsigned *word)
{
    g_last_error[0] = 0;
    if (!d || !workspace || !word) return fail(KDA_ERR_INVALID_ARG, "dims, workspace or word is NULL");
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "stream: %s", hipGetErrorString(e));
    if (d->chunk != kChunk || check_dims(d, d->num_seqs != d->batch) != KDA_OK) return KDA_ERR_INVALID_ARG;
    if (!mfma_path(d) || chunk_mfma_workspace_size(d, true, false) == 0 ||
        workspace_bytes < chunk_mfma_workspace_size(d, true, false))
        return fail(KDA_ERR_UNSUPPORTED, "this call keeps no status word");
    uint32_t w = 0;
    e = hipMemcpy(&w, static_cast<const uint8_t *>(workspace) + chunk_mfma_status_offset(d, workspace_bytes), sizeof(w),
                  hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "status read: %s", hipGetErrorString(e));
    *word = w;
    return KDA_OK;
}

kda_status kda_recurrent_step(const kda_dims *d, const void *q, const void *k, const void *v,
                              const void *log_alpha, const void *beta, float *S, void *o,
                              void *hip_stream)
{
    g_last_error[0] = 0;
    kda_status st = check_dims(d, false);
    if (st != KDA_OK) return st;
    if (d->seqlen != 1) return fail(KDA_ERR_INVALID_ARG, "recurrent step needs seqlen == 1, got %lld",
                                    (long long)d->seqlen);
    if (d->num_seqs == 0 || d->heads == 0) return KDA_OK;
    if (!q || !k || !v || !log_alpha || !beta || !S || !o)
        return fail(KDA_ERR_INVALID_ARG, "q, k, v, log_alpha, beta, S and o must be non-NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(log_alpha) || !aligned16(S) ||
        !aligned16(o) || (reinterpret_cast<uintptr_t>(beta) & 1u))
        return fail(KDA_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    return recurrent_step_dispatch(d, nullptr, nullptr, q, k, v, log_alpha, beta, S, o, nullptr, false,
                                   static_cast<hipStream_t>(hip_stream));
}

static kda_status steps_pooled_impl(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                                    const void *q, const void *k,
                                    const void *v, const void *log_alpha, const void *beta, float *S_pool,
                                    const int32_t *state_indices, void *o, void *hip_stream,
                                    bool scalar_gate = false)
{
    kda_status st = check_dims(d, false);
    if (st != KDA_OK) return st;
    if (d->seqlen < 1 || d->seqlen > recurrent_max_steps())
        return fail(KDA_ERR_INVALID_ARG, "pooled decode takes 1..%d tokens per sequence, got %lld",
                    recurrent_max_steps(), (long long)d->seqlen);
    if (d->num_seqs == 0 || d->heads == 0) return KDA_OK;
    if (!q || !k || !v || !log_alpha || !beta || !S_pool || !o)
        return fail(KDA_ERR_INVALID_ARG, "q, k, v, log_alpha, beta, S_pool and o must be non-NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || (!scalar_gate && !aligned16(log_alpha)) || !aligned16(S_pool) ||
        !aligned16(o) || (reinterpret_cast<uintptr_t>(beta) & 1u) || (reinterpret_cast<uintptr_t>(log_alpha) & 1u) ||
        (reinterpret_cast<uintptr_t>(state_indices) & 3u))
        return fail(KDA_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned (state_indices: 4)");
    return recurrent_step_dispatch(d, pro, epi, q, k, v, log_alpha, beta, S_pool, o, state_indices, scalar_gate,
                                   static_cast<hipStream_t>(hip_stream));
}

kda_status kda_recurrent_steps_pooled(const kda_dims *d, const void *q, const void *k, const void *v,
                                      const void *log_alpha, const void *beta, float *S_pool,
                                      const int32_t *state_indices, void *o, void *hip_stream)
{
    g_last_error[0] = 0;
    return steps_pooled_impl(d, nullptr, nullptr, q, k, v, log_alpha, beta, S_pool, state_indices, o, hip_stream);
}

kda_status kda_recurrent_steps_pooled_scalar_gate(const kda_dims *d, const void *q, const void *k, const void *v,
                                                  const void *log_alpha_head, const void *beta, float *S_pool,
                                                  const int32_t *state_indices, void *o, void *hip_stream)
{
    g_last_error[0] = 0;
    return steps_pooled_impl(d, nullptr, nullptr, q, k, v, log_alpha_head, beta, S_pool, state_indices, o, hip_stream,
                             true);
}

kda_status kda_recurrent_steps_fused(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                                     const void *q_raw, const void *k_raw, const void *v, const void *gate,
                                     const void *beta_logit, float *S_pool, const int32_t *state_indices,
                                     void *o, void *hip_stream)
{
    g_last_error[0] = 0;
    kda_status st = check_prologue(pro);
    if (st == KDA_OK) st = check_epilogue(epi);
    if (st != KDA_OK) return st;
    return steps_pooled_impl(d, pro, epi, q_raw, k_raw, v, gate, beta_logit, S_pool, state_indices, o, hip_stream);
}

}  // extern "C"
