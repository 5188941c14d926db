// Launch interface of the two-kernel prefill with the fused output gate (kda_prefill_gated.hip).
#pragma once
#include "kda_intra.h"

namespace kda {
namespace mfma {

struct GatedLaunch {
    const uint16_t *q, *k, *v, *log_alpha, *beta;
    const int32_t *cu;
    const float *state_in;
    float *state_out;
    void *o;
    uint8_t *ws;                    // first slot of the segment
    uint8_t *gate_ws;               // staged gate logits, kGateSlotBytes per slot
    uint32_t *status;
    const uint16_t *gate;           // gate logits [B,T,H,dv] in the input dtype
    const float *norm_w;            // RMSNorm weight [dv] or NULL (= ones)
    float rms_eps, scale;
    int64_t T, seg_chunks, seg_index, launch_chunks;
    int H, num_seqs;
    bool raw_inputs, out_bf16;
    RawParams raw;
};

kda_status launch_prefill_gated(const GatedLaunch &L, hipStream_t stream);

}  // namespace mfma
}  // namespace kda
