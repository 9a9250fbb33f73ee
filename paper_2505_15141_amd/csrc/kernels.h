// Launchers of the forward-pass kernels (internal).
#pragma once
#include "common.h"

namespace bs {

constexpr int GEMM_MAX_ROWS = 256;  // rows of x one workgroup of the many-row GEMM keeps in MFMA accumulators

struct GemmArgs {
    const void* x;        // activations [M, K]: float, or bf16 hi plane (lo plane x_plane elements further)
    size_t x_plane;
    const void* w[3];     // up to three weight matrices stacked along N
    int seg_rows[2];      // rows of segment 0 and 1 (segment 2 takes the rest); N for a single matrix
    float* out;           // split-K partials [KS][M][ldo] float32 (slice stride ks_stride elements)
    size_t ks_stride;
    int M, N, K, ldo, KS;
    int tiled;            // weights are in the 64x32-block layout written by launch_pack_weights
};

// Fused projection for a handful of rows (see gemm_dec_kernel): tiled bf16 weights, activations as planes.
constexpr int DEC_MAX_ROWS = 2;
enum { EPI_RESID = 0, EPI_QKV = 1, EPI_SWIGLU = 2 };
struct DecArgs {
    const uint16_t* xh; size_t x_plane;       // input planes [M][K] (hi; lo x_plane elements further); gemm_rows: [K/32][16][32], x_plane = 16 K
    const void* w[3]; int seg_rows[2];        // tiled matrices stacked along N (QKV), or gate and up (SWIGLU)
    int M, N, K;                              // N: output columns (per matrix for SWIGLU)
    const float* ssq_in; int ssq_tiles; float eps;     // input rows' partial sums of squares [M][ssq_tiles] (QKV, SWIGLU)
    float* x; const float* gain_next; uint16_t* out_planes; size_t out_plane; float* ssq_out;   // RESID; out_planes also SWIGLU
    int out_tiled;                            // gemm_rows: output planes in the tiled layout [N/32][16][32] (out_plane = 16 N)
    const int32_t* pos; const float2* rope; int q_len, H, KVH, hd, cache_len;                    // QKV
    float* q_out; uint16_t* k_cache; uint16_t* v_cache;
    const float* att_part; int att_splits;    // RESID with the attention's per-split partials as input instead of planes (uses H, hd)
};
bool gemm_dec_fits(int M, int K);
int launch_gemm_dec(int epi, const DecArgs& a, hipStream_t s);
// The same epilogues (EPI_QKV, EPI_SWIGLU) for up to 16 rows of a wide model: one workgroup per compute unit owns several
// 16-column units over the whole K.  gemm_rows_units: units per workgroup at most (0: the kernel does not apply), *grid: workgroups.
int gemm_rows_units(int epi, int M, int N, int K, int* grid);
int launch_gemm_rows(int epi, const DecArgs& a, hipStream_t s);
int launch_embed_dec(const int32_t* tok, const void* embed, const float* gain, int M, int d, float* x, void* planes,
                     size_t plane, float* ssq, hipStream_t s);

// One resident kernel for a whole forward pass over one or two rows of a small model (see step.hip).
constexpr int STEP_MAXL = 16;            // layers whose pointers travel as kernel arguments
struct StepArgs {
    const uint16_t* w[STEP_MAXL][7];     // tiled wq wk wv wo w_gate w_up w_down
    const float* an[STEP_MAXL];          // attention / feed-forward norm gains
    const float* fn[STEP_MAXL];
    const uint16_t* embed; const float* final_norm; const uint16_t* lm_head;
    int n_layers, d, H, KVH, hd, ff, V; float eps;
    int B, q_len, M, logit_rows;
    const int32_t* pos; const int32_t* tok; const float2* rope;      // written by the prep kernel
    char* kv; size_t kv_layer; int cache_len;
    void *X, *Q, *KVN, *PA, *ACT;        // exchange buffers of 8-byte cells {value, flag}: residual [copies][M][d], queries [M][nq],
                                         // new keys|values [M][2 nkv], attention partials [M][H][splits + 1][hd + 4] (the last slot:
                                         // the keys of the pass's own rows), SwiGLU output [M][ff]; every flag is zero when the
                                         // kernel starts (the prep kernel clears them)
    int32_t* status; int splits;
    float* logits; size_t logits_bstride;
    unsigned spin_limit;                 // polls of a cell before a workgroup gives up (status bit 16)
    int kp;                              // set by the launcher: padded row of the staged planes
};
bool step_fits(const bs_model_cfg& c, int B, int q_len, int n_layers);
// splits of the cached keys the resident step uses for B sequences and this cache length; 0: no room for the units
int step_splits(const bs_model_cfg& c, int B, int max_len);
// bytes of the exchange buffers X, Q, KVN, PA, ACT (each 256-byte aligned, in this order; off[i] = where buffer i starts)
size_t step_exchange_bytes(const bs_model_cfg& c, int M, int splits, size_t off[5]);
int step_grid();                         // workgroups of the resident kernel = compute units of the device
int launch_step(const StepArgs& a, hipStream_t s);

int gemm_splits(int dtype, int N, int K, int M);
int profile_enable(int on);
int profile_collect(int mt_filter, double* total_ms, double* total_bytes, long long* launches);
int launch_gemm(int dtype, GemmArgs a, hipStream_t s);
size_t packed_elems(int N, int K);                       // elements of the tiled copy of an [N][K] matrix
int launch_pack_weights(const void* src, void* dst, int N, int K, hipStream_t s);

// clear_bytes > 0: also zeroes that many bytes at `clear` (a multiple of 16, 16-byte aligned): the exchange cells of the
// resident step kernel that follows
int launch_prep(const int32_t* q_tokens, int q_stride, const int32_t* kv_len, int kv_base, int B, int q_len,
                int max_len, int V, int hd, float rope_base, int32_t* pos, int32_t* tok, float2* rope,
                int32_t* status, void* clear, size_t clear_bytes, hipStream_t s);
int launch_embed(int dtype, const int32_t* tok, const void* embed, int M, int d, float* x, hipStream_t s);
int launch_rmsnorm(int dtype, float* x, const float* pend, int pend_ks, size_t pend_stride, const float* gain, int d,
                   float eps, int n_seq, int rows_in, int rows_out, size_t plane, void* out, hipStream_t s);
// bf16 models: residual completion + planes of gain .* x + per-chunk sums of squares [rows][norm_chunks(d)]; the
// consumers below apply the rows' RMS scale when given those sums (ssq != nullptr)
int norm_chunks(int d);
// tiled: planes in the layout of the whole-K projections for up to 16 rows, [d/32][16][32], plane = 16*d elements
int launch_resid_sum(float* x, const float* pend, int pend_ks, size_t pend_stride, const float* gain, int d, int rows,
                     size_t plane, void* out, float* ssq, bool tiled, hipStream_t s);
int launch_swiglu(int dtype, const float* part, int ks, size_t ks_stride, int M, int ff, size_t plane, void* out,
                  const float* ssq, int d, float eps, hipStream_t s);
int launch_rope_kv(int dtype, const float* part, int ks, size_t ks_stride, const int32_t* pos, const float2* rope, int M,
                   int q_len, int H, int KVH, int hd, int max_len, float* q_out, void* k_cache, void* v_cache,
                   const float* ssq, int d, float eps, hipStream_t s);
// out == nullptr: the splits are left un-merged in `part` (the consumer combines them)
// Exchange cells for combining the key splits inside the attention kernel (at most 16 query rows per head group, all
// workgroups resident together; otherwise a merge kernel runs): zero when the pass starts, one flag per layer.
struct AttnCells { void* buf; size_t bytes; unsigned flag, spin_limit; int32_t* status; };
size_t attn_cells_bytes(int rows, int H, int hd, int n_splits);
int launch_attention(int dtype, const float* q, const void* k_cache, const void* v_cache, const int32_t* pos, int B,
                     int q_len, int H, int KVH, int hd, int max_len, int n_splits, float* part, size_t plane, void* out, bool out_tiled, const AttnCells* cells,
                     hipStream_t s);

}  // namespace bs
