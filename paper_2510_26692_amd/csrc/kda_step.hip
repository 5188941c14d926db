// Recurrent decode step of KDA (Section 3, Eq. (1); Section 6.3 "Inference
// strategy"): one new token per (sequence, head), fp32 state updated in place.
//
//     S <- Diag(alpha) S;  r = v - S^T k;  S <- S + beta k r^T;  o = scale S^T q
//
// The step is pure streaming: each dk x dv fp32 state is read once and written
// once (64 KiB each way at dk = dv = 128) for ~0.9 FLOP per byte, so the kernel
// is laid out for HBM, not for the matrix cores.  Every column of S is an
// independent recurrence, so a wavefront owns a 32-column slice of one state and
// never talks to another wavefront: lanes are arranged 8 (row groups) x 8
// (float4 column groups), each lane keeps dk/8 float4 of the slice in
// registers, the two reductions over dk finish with three xor-shuffles, and the
// slice is written back from the same registers.  A block is the dv/32
// wavefronts of one (sequence, head), so a block streams one contiguous state.
#include "kda_common.h"

namespace kda {

// steps:   tokens per sequence handled by one launch (1 = plain decode; up to kMaxSteps for
//          multi-token steps such as speculative verification): the state is read once, taken
//          through the tokens in order in registers, and written once.
// indices: NULL, or one state-pool slot per sequence (sequence n works on state indices[n];
//          a negative entry skips the sequence).
constexpr int kMaxSteps = 8;

// kRaw:    q, k, log_alpha, beta are the raw projections of Section 4; the kernel applies L2Norm,
//          Sigmoid and log alpha = -a_scale[h] softplus(gate + dt_bias[h][c]) while it stages them.
// kEpi:    o leaves as Sigmoid(out_gate) * RMSNorm(o) * norm_w (Section 4, output gate); the mean
//          square runs over the DV values of the (token, head), i.e. over the block's waves.
template <typename Tin, int DK, int DV, bool kRaw, bool kEpi>
__global__ __launch_bounds__(DV * 2)
void kda_step_kernel(const Tin *__restrict__ q, const Tin *__restrict__ k,
                     const Tin *__restrict__ v, const Tin *__restrict__ log_alpha,
                     const Tin *__restrict__ beta, float *__restrict__ S,
                     void *__restrict__ o, int o_bf16, int alpha_per_head, float scale, int H, int steps,
                     const int32_t *__restrict__ indices, const float *__restrict__ a_scale,
                     const float *__restrict__ dt_bias, float l2_eps, const Tin *__restrict__ out_gate,
                     const float *__restrict__ norm_w, float rms_eps)
{
    constexpr int ROWS = DK / 8;             // state rows per lane
    __shared__ float s_alpha[kMaxSteps][DK], s_k[kMaxSteps][DK], s_q[kMaxSteps][DK];
    __shared__ float s_ssq[kMaxSteps][DV / 32];

    const int64_t pair = blockIdx.x;         // (sequence, head) index
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int cg = lane & 7;                 // float4 column group inside the slice
    const int rg = lane >> 3;                // row group: rows rg, rg+8, ...
    const int col = wave * 32 + cg * 4;

    const int64_t n = pair / H;
    const int h = (int)(pair - n * H);
    int64_t state = pair;                    // which dk x dv state this block works on
    if (indices) {
        const int32_t slot = indices[n];
        if (slot < 0) return;                // uniform for the block
        state = (int64_t)slot * H + h;
    }
    // token t of this pair: element offset (n * steps + t) * H + h in units of one head row
    const int64_t row0 = n * steps * H + h;

    // Token vectors: decay, key and query are needed per row by every lane.
    if (!kRaw) {
        for (int i = tid; i < steps * DK; i += DV * 2) {
            const int t = i / DK, c = i - t * DK;
            const int64_t off = (row0 + (int64_t)t * H) * DK + c;
            // (alpha_per_head: log_alpha is [N,steps,H], one decay for all channels of a head)
            s_alpha[t][c] = fast_exp2(load_as_float(log_alpha + (alpha_per_head ? row0 + (int64_t)t * H : off)) * kLog2e);
            s_k[t][c] = load_as_float(k + off);
            s_q[t][c] = load_as_float(q + off);
        }
    } else {
        // one wave per token: a lane holds channels lane, lane + 64, ...; the norms are wave sums
        const float as = a_scale ? a_scale[h] : 1.f;
        for (int t = wave; t < steps; t += DV / 32) {
            const int64_t off = (row0 + (int64_t)t * H) * DK;
            float qv[DK / 64], kv[DK / 64], sq = 0.f, sk = 0.f;
#pragma unroll
            for (int j = 0; j < DK / 64; ++j) {
                const int c = lane + 64 * j;
                qv[j] = load_as_float(q + off + c); kv[j] = load_as_float(k + off + c);
                sq = fmaf(qv[j], qv[j], sq); sk = fmaf(kv[j], kv[j], sk);
                const float x = load_as_float(log_alpha + off + c) + (dt_bias ? dt_bias[h * DK + c] : 0.f);
                const float tt = x * kLog2e;
                const float sp = (tt > 30.f) ? tt : __log2f(1.f + fast_exp2(tt));   // log2(1 + e^x)
                s_alpha[t][c] = fast_exp2(-as * sp);
            }
#pragma unroll
            for (int dd = 1; dd < 64; dd <<= 1) { sq += __shfl_xor(sq, dd); sk += __shfl_xor(sk, dd); }
            const float iq = __builtin_amdgcn_rsqf(sq + l2_eps), ik = __builtin_amdgcn_rsqf(sk + l2_eps);
#pragma unroll
            for (int j = 0; j < DK / 64; ++j) {
                s_q[t][lane + 64 * j] = qv[j] * iq;
                s_k[t][lane + 64 * j] = kv[j] * ik;
            }
        }
    }

    // Stream the slice in: ROWS independent 16-byte loads per lane.
    f32x4 *Sp = reinterpret_cast<f32x4 *>(S + state * (int64_t)(DK * DV) + (int64_t)rg * DV + col);
    f32x4 s[ROWS];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) s[m] = __builtin_nontemporal_load(Sp + (int64_t)m * (8 * DV / 4));

    __syncthreads();

    for (int t = 0; t < steps; ++t) {
        const int64_t row = row0 + (int64_t)t * H;
        float vv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) vv[c] = load_as_float(v + row * DV + col + c);
        float b = load_as_float(beta + row);
        if (kRaw) b = __builtin_amdgcn_rcpf(1.f + fast_exp2(-b * kLog2e));          // Sigmoid
        const bool last = t + 1 == steps;

        // Decay, then the memory's prediction S^T k for this lane's columns.
        float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
#pragma unroll
        for (int m = 0; m < ROWS; ++m) {
            const float a = s_alpha[t][rg + 8 * m];
            const float kk = s_k[t][rg + 8 * m];
            s[m].x *= a; s[m].y *= a; s[m].z *= a; s[m].w *= a;
            p0 = fmaf(kk, s[m].x, p0); p1 = fmaf(kk, s[m].y, p1);
            p2 = fmaf(kk, s[m].z, p2); p3 = fmaf(kk, s[m].w, p3);
        }
#pragma unroll
        for (int d = 8; d < 64; d <<= 1) {
            p0 += __shfl_xor(p0, d); p1 += __shfl_xor(p1, d);
            p2 += __shfl_xor(p2, d); p3 += __shfl_xor(p3, d);
        }
        // w = beta * (v - S^T k): the delta-rule correction written along k.
        const float w0 = b * (vv[0] - p0), w1 = b * (vv[1] - p1);
        const float w2 = b * (vv[2] - p2), w3 = b * (vv[3] - p3);

        float o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
#pragma unroll
        for (int m = 0; m < ROWS; ++m) {
            const float kk = s_k[t][rg + 8 * m];
            const float qq = s_q[t][rg + 8 * m];
            s[m].x = fmaf(kk, w0, s[m].x); s[m].y = fmaf(kk, w1, s[m].y);
            s[m].z = fmaf(kk, w2, s[m].z); s[m].w = fmaf(kk, w3, s[m].w);
            o0 = fmaf(qq, s[m].x, o0); o1 = fmaf(qq, s[m].y, o1);
            o2 = fmaf(qq, s[m].z, o2); o3 = fmaf(qq, s[m].w, o3);
            if (last) __builtin_nontemporal_store(s[m], Sp + (int64_t)m * (8 * DV / 4));
        }
#pragma unroll
        for (int d = 8; d < 64; d <<= 1) {
            o0 += __shfl_xor(o0, d); o1 += __shfl_xor(o1, d);
            o2 += __shfl_xor(o2, d); o3 += __shfl_xor(o3, d);
        }
        o0 *= scale; o1 *= scale; o2 *= scale; o3 *= scale;
        if (kEpi) {
            // every lane holds the four outputs of its column group: sum the squares over the
            // wave's eight groups, then over the block's waves through LDS
            float ssq = o0 * o0 + o1 * o1 + o2 * o2 + o3 * o3;
            ssq += __shfl_xor(ssq, 1); ssq += __shfl_xor(ssq, 2); ssq += __shfl_xor(ssq, 4);
            if (lane == 0) s_ssq[t][wave] = ssq;
            __syncthreads();
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < DV / 32; ++w) tot += s_ssq[t][w];
            const float rstd = __builtin_amdgcn_rsqf(tot * (1.0f / DV) + rms_eps);
            float gv[4], wv[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                gv[c] = load_as_float(out_gate + row * DV + col + c);
                wv[c] = norm_w ? norm_w[col + c] : 1.f;
            }
            o0 *= rstd * wv[0] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-gv[0] * kLog2e));
            o1 *= rstd * wv[1] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-gv[1] * kLog2e));
            o2 *= rstd * wv[2] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-gv[2] * kLog2e));
            o3 *= rstd * wv[3] * __builtin_amdgcn_rcpf(1.f + fast_exp2(-gv[3] * kLog2e));
        }
        if (rg == 0) {
            if (o_bf16) {
                const uint32_t lo = pack_bf16x2(o0, o1), hi = pack_bf16x2(o2, o3);
                uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<uint16_t *>(o) + row * DV + col);
                dst[0] = lo; dst[1] = hi;
            } else {
                f32x4 out = {o0, o1, o2, o3};
                *reinterpret_cast<f32x4 *>(static_cast<float *>(o) + row * DV + col) = out;
            }
        }
    }
}

template <typename Tin, int DK, int DV>
static kda_status launch_step(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                              const void *q, const void *k, const void *v, const void *log_alpha,
                              const void *beta, float *S, void *o, const int32_t *indices, bool scalar_gate,
                              hipStream_t stream)
{
    const int64_t pairs = (int64_t)d->num_seqs * d->heads;
    if (pairs == 0) return KDA_OK;
    if (pairs > 0x7fffffffLL) return fail(KDA_ERR_INVALID_ARG, "num_seqs*heads exceeds 2^31-1");
    auto step = pro ? (epi ? kda_step_kernel<Tin, DK, DV, true, true> : kda_step_kernel<Tin, DK, DV, true, false>)
                    : (epi ? kda_step_kernel<Tin, DK, DV, false, true> : kda_step_kernel<Tin, DK, DV, false, false>);
    hipLaunchKernelGGL(step, dim3((unsigned)pairs), dim3(DV * 2), 0, stream,
                       static_cast<const Tin *>(q), static_cast<const Tin *>(k),
                       static_cast<const Tin *>(v), static_cast<const Tin *>(log_alpha),
                       static_cast<const Tin *>(beta), S, o, (int)(d->out_dtype == KDA_BF16), (int)scalar_gate, d->scale,
                       (int)d->heads, (int)d->seqlen, indices, pro ? pro->a_scale : nullptr,
                       pro ? pro->dt_bias : nullptr, pro ? pro->l2norm_eps : 0.f,
                       static_cast<const Tin *>(epi ? epi->gate : nullptr), epi ? epi->norm_weight : nullptr,
                       epi ? epi->rms_eps : 0.f);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KDA_ERR_LAUNCH, "kda_step_kernel: %s", hipGetErrorString(e));
    return KDA_OK;
}

int recurrent_max_steps() { return kMaxSteps; }

kda_status recurrent_step_dispatch(const kda_dims *d, const kda_prologue *pro, const kda_epilogue *epi,
                                   const void *q, const void *k, const void *v, const void *log_alpha,
                                   const void *beta, float *S, void *o, const int32_t *indices, bool scalar_gate,
                                   hipStream_t stream)
{
    const bool bf = d->in_dtype == KDA_BF16;
    if (d->dk == 128 && d->dv == 128)
        return bf ? launch_step<__hip_bfloat16, 128, 128>(d, pro, epi, q, k, v, log_alpha, beta, S, o, indices, scalar_gate, stream)
                  : launch_step<float, 128, 128>(d, pro, epi, q, k, v, log_alpha, beta, S, o, indices, scalar_gate, stream);
    if (d->dk == 64 && d->dv == 64)
        return bf ? launch_step<__hip_bfloat16, 64, 64>(d, pro, epi, q, k, v, log_alpha, beta, S, o, indices, scalar_gate, stream)
                  : launch_step<float, 64, 64>(d, pro, epi, q, k, v, log_alpha, beta, S, o, indices, scalar_gate, stream);
    return fail(KDA_ERR_UNSUPPORTED, "recurrent step supports dk == dv in {64,128}, got %d x %d",
                d->dk, d->dv);
}

}  // namespace kda
