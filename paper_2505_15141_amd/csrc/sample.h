// Launchers of the sampling kernels, shared with the round driver (internal).
#pragma once
#include "common.h"

namespace bs {

struct DrawParams {
    const float* logits;     // [B, row_stride] float32, first V entries of each row are used
    int row_stride, V;
    float inv_temp;
    uint64_t seed;
    const uint32_t* round_ptr;   // device round counter (overrides `round` when non-null)
    uint32_t round, slot;
    // up to three destinations: out[b * stride + off] = token
    int32_t* out0; int stride0, off0;
    int32_t* out1; int stride1, off1;
    int32_t* out2; int stride2, off2;
};

int launch_draw(const DrawParams& a, int B, hipStream_t stream);

int launch_spec_rows(const void* p_logits, const void* q_logits, const int32_t* draft_tokens, int B, int gamma, int V,
                     int dtype, float temperature, const float* uniforms, uint64_t seed, const uint32_t* round_ptr,
                     uint32_t round, int32_t* flags, int32_t* cand, float* margins, hipStream_t stream);

int launch_spec_resolve(const int32_t* flags, const int32_t* cand, int B, int gamma, int32_t* accept_len,
                        int32_t* next_token, hipStream_t stream);

}  // namespace bs
