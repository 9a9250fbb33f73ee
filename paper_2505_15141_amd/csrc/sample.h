// Launchers of the sampling kernels, shared with the round driver (internal).
#pragma once
#include "common.h"

namespace bs {

struct DrawParams {
    const float* logits;     // [B, row_stride] float32, first V entries of each row are used
    int row_stride, V;
    float inv_temp;
    int greedy;              // 1: token = argmax of the row (temperature 0), no uniform used
    uint64_t seed;
    const uint32_t* round_ptr;   // device round counter (overrides `round` when non-null)
    uint32_t round, slot;
    // up to three destinations: out[b * stride + off] = token
    int32_t* out0; int stride0, off0;
    int32_t* out1; int stride1, off1;
    int32_t* out2; int stride2, off2;
};

int launch_draw(const DrawParams& a, int B, hipStream_t stream);

// Scratch for the per-row softmax statistics of one sampling call.
size_t spec_scratch_bytes(int B, int gamma);

// Accept/reject + residual/bonus draw.  flags/cand [B, gamma+1] (round driver) and accept_len/next_token [B]
// (stand-alone call) are optional outputs.
int launch_spec_sample(const void* p_logits, const void* q_logits, const int32_t* draft_tokens, int B, int gamma, int V,
                       int dtype, float temperature, const float* uniforms, uint64_t seed, const uint32_t* round_ptr,
                       uint32_t round, void* stats_scratch, int32_t* flags, int32_t* cand, int32_t* accept_len,
                       int32_t* next_token, float* margins, hipStream_t stream);

}  // namespace bs
