// Launchers of the forward-pass kernels (internal).
#pragma once
#include "common.h"

namespace bs {

constexpr int GEMM_MAX_ROWS = 96;   // rows of x one bf16 GEMM launch keeps in MFMA accumulators

enum { GEMM_STORE = 0, GEMM_ADD = 1, GEMM_SWIGLU = 2 };

struct GemmArgs {
    const void* x;        // [M, K] storage dtype
    const void* w[3];     // weight segments stacked along N (STORE/ADD), or {gate, up} (SWIGLU)
    int seg_rows[2];      // rows of segment 0 and 1 (segment 2 takes the rest); N for a single matrix
    void* out;            // STORE/ADD: float32 [M, ldo]; SWIGLU: storage dtype [M, ldo]
    int M, N, K, ldo;
};

int launch_gemm(int dtype, int epi, GemmArgs a, hipStream_t s);

int launch_prep(const int32_t* q_tokens, int q_stride, const int32_t* kv_len, int kv_base, int B, int q_len,
                int max_len, int V, int hd, float rope_base, int32_t* pos, int32_t* tok, float2* rope,
                int32_t* status, hipStream_t s);
int launch_embed(int dtype, const int32_t* tok, const void* embed, int M, int d, float* x, hipStream_t s);
int launch_rmsnorm(int dtype, const float* x, const float* gain, int d, float eps, int n_seq, int rows_in,
                   int rows_out, void* out, hipStream_t s);
int launch_rope_kv(int dtype, const float* qkv, const int32_t* pos, const float2* rope, int M, int q_len, int H,
                   int KVH, int hd, int max_len, void* q_out, void* k_cache, void* v_cache, hipStream_t s);
int launch_attention(int dtype, const void* q, const void* k_cache, const void* v_cache, const int32_t* pos, int B,
                     int q_len, int H, int KVH, int hd, int max_len, int n_splits, float* part, void* out,
                     hipStream_t s);

}  // namespace bs
