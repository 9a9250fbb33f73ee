// Device kernels of the transformer forward used by the verification pass (App. A: the target model
// scores all gamma+1 positions in one pass) and by the draft model's steps.
//
//   prep        positions, clamped tokens, RoPE cos/sin table, overflow status
//   embed       token embedding -> fp32 residual stream
//   rmsnorm     fp32 residual -> normalised activations in the storage dtype
//   gemm        y = x W^T: bf16 weights streamed once from HBM through MFMA 16x16x32 tiles (the
//               contraction is skinny: M = B*(gamma+1) rows, so it is bound by weight bandwidth),
//               fp32 variant for the fp32 plumbing configuration
//   rope_kv     rotate q and k, write k/v into the cache
//   attention   q_len causal query rows per head against the contiguous KV cache, split along the
//               keys with online softmax; merge kernel combines the splits
#include <math.h>
#include "common.h"
#include "kernels.h"

namespace bs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- storage dtype helpers ----------------------------------------------------------------------
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
template <typename T> __device__ __forceinline__ T from_f(float f);
template <> __device__ __forceinline__ float from_f<float>(float f) { return f; }
template <> __device__ __forceinline__ uint16_t from_f<uint16_t>(float f) {   // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- prep ---------------------------------------------------------------------------------------
// One workgroup per sequence.  pos[m] = kv_len[b] + kv_base + j, or -1 for a sequence that would run
// past max_len (then nothing of it is written anywhere).  tok[m] = token clamped into [0, V).
__global__ void prep_kernel(const int32_t* __restrict__ q_tokens, int q_stride, const int32_t* __restrict__ kv_len,
                            int kv_base, int q_len, int max_len, int V, int half_hd, float rope_base,
                            int32_t* __restrict__ pos, int32_t* __restrict__ tok, float2* __restrict__ rope,
                            int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int kvl = (kv_len ? kv_len[b] : 0) + kv_base;
    const bool ok = kvl >= 0 && kvl + q_len <= max_len;
    if (!ok && threadIdx.x == 0) atomicOr(status, 1);
    for (int j = threadIdx.x; j < q_len; j += blockDim.x) {
        const int m = b * q_len + j;
        int t = q_tokens[(size_t)b * q_stride + j];
        if (t < 0 || t >= V) { t = 0; atomicOr(status, 2); }
        tok[m] = t;
        pos[m] = ok ? kvl + j : -1;
    }
    for (int idx = threadIdx.x; idx < q_len * half_hd; idx += blockDim.x) {
        const int j = idx / half_hd, i = idx % half_hd;
        const double inv_freq = pow((double)rope_base, -(double)i / (double)half_hd);   // base^(-2i/hd)
        const double ang = (double)(ok ? kvl + j : 0) * inv_freq;
        double s, c;
        sincos(ang, &s, &c);
        rope[(size_t)(b * q_len + j) * half_hd + i] = make_float2((float)c, (float)s);
    }
}

// ---- embedding ----------------------------------------------------------------------------------
template <typename T>
__global__ void embed_kernel(const int32_t* __restrict__ tok, const T* __restrict__ embed, int d, float* __restrict__ x) {
    const int m = blockIdx.x;
    const T* row = embed + (size_t)tok[m] * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = to_f(row[i]);
}

// ---- RMSNorm ------------------------------------------------------------------------------------
// out row r takes input row (r / rows_out) * rows_in + (rows_in - rows_out) + r % rows_out
// (rows_out = rows_in: identity; rows_out < rows_in: the trailing rows of every sequence).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      int d, float eps, int rows_in, int rows_out,
                                                      T* __restrict__ out) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    const int src = (r / rows_out) * rows_in + (rows_in - rows_out) + r % rows_out;
    const float* row = x + (size_t)src * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) { const float v = row[i]; ss += v * v; }
    ss = wsum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) out[(size_t)r * d + i] = from_f<T>(row[i] * scale * gain[i]);
}

// ---- GEMM, bf16 MFMA, weight streaming -------------------------------------------------------------
// y[m][n] = sum_k x[m][k] * W[n][k].  One workgroup = 4 wavefronts owns 16 output columns n (16 weight
// rows) and every one of the M <= 16*MT rows; the wavefronts split K in interleaved 128-element chunks
// and reduce through LDS.  Weight tile -> MFMA A operand (lane = (row l%16, k-slot l/16), 16-byte loads
// straight from HBM), activations -> B operand (L2-resident).  Up to three weight segments stacked along
// n (fused q/k/v projection) or a gate/up pair with the SwiGLU epilogue.
enum { EPI_STORE = 0, EPI_ADD = 1, EPI_SWIGLU = 2 };

__device__ __forceinline__ uint4 ldg16(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }

template <int MT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs a) {
    constexpr int NACC = (EPI == EPI_SWIGLU) ? 2 : 1;
    __shared__ float red[4][NACC * MT][64][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int n0 = blockIdx.x * 16;
    // weight rows of this tile (segment lookup; tiles never straddle segments because every segment's row
    // count is a multiple of 16 - checked on the host)
    const uint16_t* w0;
    const uint16_t* w1 = nullptr;
    {
        int n = n0 + li;
        if (n >= a.N) n = a.N - 1;
        if (EPI == EPI_SWIGLU) {
            w0 = reinterpret_cast<const uint16_t*>(a.w[0]) + (size_t)n * a.K;
            w1 = reinterpret_cast<const uint16_t*>(a.w[1]) + (size_t)n * a.K;
        } else {
            int seg = 0, local = n;
            if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
            w0 = reinterpret_cast<const uint16_t*>(a.w[seg]) + (size_t)local * a.K;
        }
    }
    const uint16_t* x = reinterpret_cast<const uint16_t*>(a.x);
    f32x4 acc[NACC][MT];
#pragma unroll
    for (int s = 0; s < NACC; ++s)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[s][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = (a.K + 127) / 128;
    for (int c = wave; c < nchunks; c += 4) {
        const int kb = c * 128 + lq * 8;
        uint4 wa[4], wb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = kb + j * 32;
            const bool ok = k < a.K;                      // K % 8 == 0 (host check): whole 16-byte groups
            wa[j] = ok ? ldg16(w0 + k) : make_uint4(0, 0, 0, 0);
            if (EPI == EPI_SWIGLU) wb[j] = ok ? ldg16(w1 + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = t * 16 + li;
            uint4 xv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = kb + j * 32;
                xv[j] = (m < a.M && k < a.K) ? ldg16(x + (size_t)m * a.K + k) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bf16x8 B = __builtin_bit_cast(bf16x8, xv[j]);
                acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[j]), B, acc[0][t], 0, 0, 0);
                if (EPI == EPI_SWIGLU)
                    acc[1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wb[j]), B, acc[1][t], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int s = 0; s < NACC; ++s)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[wave][s * MT + t][lane][e] = acc[s][t][e];
    __syncthreads();
    // thread -> (e = wave, lane): D[n = 4*(lane/16)+e][m = lane%16] of every m-tile
    const int e = wave;
    const int n = n0 + 4 * lq + e;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = t * 16 + li;
        float v0 = red[0][t][lane][e] + red[1][t][lane][e] + red[2][t][lane][e] + red[3][t][lane][e];
        if (m >= a.M || n >= a.N) continue;
        if (EPI == EPI_SWIGLU) {
            const float up = red[0][MT + t][lane][e] + red[1][MT + t][lane][e] + red[2][MT + t][lane][e] + red[3][MT + t][lane][e];
            const float act = v0 / (1.0f + __expf(-v0)) * up;
            reinterpret_cast<uint16_t*>(a.out)[(size_t)m * a.ldo + n] = from_f<uint16_t>(act);
        } else if (EPI == EPI_ADD) {
            float* o = reinterpret_cast<float*>(a.out) + (size_t)m * a.ldo + n;
            *o += v0;
        } else {
            reinterpret_cast<float*>(a.out)[(size_t)m * a.ldo + n] = v0;
        }
    }
}

// ---- GEMM, fp32 (plumbing configuration) ----------------------------------------------------------
// One wavefront per output column n, lanes stride K, 8 rows of x at a time.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    if (n >= a.N) return;
    const float* w0;
    const float* w1 = nullptr;
    if (EPI == EPI_SWIGLU) {
        w0 = reinterpret_cast<const float*>(a.w[0]) + (size_t)n * a.K;
        w1 = reinterpret_cast<const float*>(a.w[1]) + (size_t)n * a.K;
    } else {
        int seg = 0, local = n;
        if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
        w0 = reinterpret_cast<const float*>(a.w[seg]) + (size_t)local * a.K;
    }
    const float* x = reinterpret_cast<const float*>(a.x);
    for (int m0 = 0; m0 < a.M; m0 += 8) {
        float acc0[8], acc1[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
        for (int k = lane; k < a.K; k += 64) {
            const float wv = w0[k];
            const float uv = (EPI == EPI_SWIGLU) ? w1[k] : 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float xv = (m0 + r < a.M) ? x[(size_t)(m0 + r) * a.K + k] : 0.f;
                acc0[r] = fmaf(xv, wv, acc0[r]);
                if (EPI == EPI_SWIGLU) acc1[r] = fmaf(xv, uv, acc1[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float v0 = wsum(acc0[r]);
            const float v1 = (EPI == EPI_SWIGLU) ? wsum(acc1[r]) : 0.f;
            if (lane == 0 && m0 + r < a.M) {
                float* o = reinterpret_cast<float*>(a.out) + (size_t)(m0 + r) * a.ldo + n;
                if (EPI == EPI_SWIGLU) *o = v0 / (1.0f + __expf(-v0)) * v1;
                else if (EPI == EPI_ADD) *o += v0;
                else *o = v0;
            }
        }
    }
}

template <int EPI>
static int launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
    const dim3 grid((a.N + 15) / 16), block(256);
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) hipLaunchKernelGGL((gemm_bf16_kernel<1, EPI>), grid, block, 0, s, a);
    else if (mt <= 2) hipLaunchKernelGGL((gemm_bf16_kernel<2, EPI>), grid, block, 0, s, a);
    else if (mt <= 4) hipLaunchKernelGGL((gemm_bf16_kernel<4, EPI>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((gemm_bf16_kernel<6, EPI>), grid, block, 0, s, a);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_gemm(int dtype, int epi, GemmArgs a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return BS_OK;
    if (dtype == BS_F32) {
        const dim3 grid((a.N + 3) / 4), block(256);
        if (epi == EPI_STORE) hipLaunchKernelGGL((gemm_f32_kernel<EPI_STORE>), grid, block, 0, s, a);
        else if (epi == EPI_ADD) hipLaunchKernelGGL((gemm_f32_kernel<EPI_ADD>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((gemm_f32_kernel<EPI_SWIGLU>), grid, block, 0, s, a);
        BS_LAUNCH_CHECK();
        return BS_OK;
    }
    // bf16: at most GEMM_MAX_ROWS rows per launch (accumulators live in registers)
    const size_t xrow = (size_t)a.K * 2;
    const size_t orow = (size_t)a.ldo * (epi == EPI_SWIGLU ? 2 : 4);
    for (int m0 = 0; m0 < a.M; m0 += GEMM_MAX_ROWS) {
        GemmArgs c = a;
        c.M = (a.M - m0 < GEMM_MAX_ROWS) ? a.M - m0 : GEMM_MAX_ROWS;
        c.x = reinterpret_cast<const char*>(a.x) + (size_t)m0 * xrow;
        c.out = reinterpret_cast<char*>(a.out) + (size_t)m0 * orow;
        int rc;
        if (epi == EPI_STORE) rc = launch_gemm_bf16<EPI_STORE>(c, s);
        else if (epi == EPI_ADD) rc = launch_gemm_bf16<EPI_ADD>(c, s);
        else rc = launch_gemm_bf16<EPI_SWIGLU>(c, s);
        if (rc != BS_OK) return rc;
    }
    return BS_OK;
}

// ---- RoPE + KV append -----------------------------------------------------------------------------
// grid (M, H + 2*KVH); thread = one rotation pair.  qkv row layout: [q heads | k heads | v heads].
template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ qkv, const int32_t* __restrict__ pos,
                               const float2* __restrict__ rope, int q_len, int H, int KVH, int hd, int max_len,
                               T* __restrict__ q_out, T* __restrict__ k_cache, T* __restrict__ v_cache) {
    const int m = blockIdx.x, head = blockIdx.y, i = threadIdx.x;       // i < hd/2
    const int p = pos[m];
    const int b = m / q_len;
    const int ld = (H + 2 * KVH) * hd;
    const float* src = qkv + (size_t)m * ld + (size_t)head * hd;
    const float x0 = src[2 * i], x1 = src[2 * i + 1];
    if (head < H + KVH) {
        const float2 cs = rope[(size_t)m * (hd / 2) + i];
        const float r0 = x0 * cs.x - x1 * cs.y, r1 = x0 * cs.y + x1 * cs.x;
        if (head < H) {
            T* dst = q_out + (size_t)m * H * hd + (size_t)head * hd;
            dst[2 * i] = from_f<T>(r0); dst[2 * i + 1] = from_f<T>(r1);
        } else if (p >= 0) {
            T* dst = k_cache + (((size_t)b * KVH + (head - H)) * max_len + p) * hd;
            dst[2 * i] = from_f<T>(r0); dst[2 * i + 1] = from_f<T>(r1);
        }
    } else if (p >= 0) {
        T* dst = v_cache + (((size_t)b * KVH + (head - H - KVH)) * max_len + p) * hd;
        dst[2 * i] = from_f<T>(x0); dst[2 * i + 1] = from_f<T>(x1);
    }
}

// ---- attention -------------------------------------------------------------------------------------
// grid (n_splits, H, B), 256 lanes.  The keys 0..n_keys-1 (n_keys = pos of the last query row + 1) are cut
// into n_splits chunks of whole 64-key tiles; the 4 wavefronts of a workgroup take the tiles of their
// chunk in turn.  Score phase: lane = key.  Value phase: lane = head-dim element (d and d+64).
// Query rows are handled ATT_RB at a time.  Writes un-normalised partials (m, l, o[hd]) per split.
constexpr int ATT_RB = 9;

template <typename T>
__device__ __forceinline__ void load8(const T* p, float out[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float out[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float out[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    out[0] = __uint_as_float(a.x << 16); out[1] = __uint_as_float(a.x & 0xFFFF0000u);
    out[2] = __uint_as_float(a.y << 16); out[3] = __uint_as_float(a.y & 0xFFFF0000u);
    out[4] = __uint_as_float(a.z << 16); out[5] = __uint_as_float(a.z & 0xFFFF0000u);
    out[6] = __uint_as_float(a.w << 16); out[7] = __uint_as_float(a.w & 0xFFFF0000u);
}

template <typename T>
__global__ __launch_bounds__(256) void attn_kernel(const T* __restrict__ q, const T* __restrict__ k_cache,
                                                   const T* __restrict__ v_cache, const int32_t* __restrict__ pos,
                                                   int q_len, int H, int KVH, int hd, int max_len, float scale,
                                                   float* __restrict__ part) {
    __shared__ float qs[ATT_RB][128];            // scaled query rows
    __shared__ float ps[4][ATT_RB][64];          // per-wavefront probabilities of the current tile
    __shared__ float wm[4][ATT_RB], wl[4][ATT_RB];
    __shared__ float wo[4][ATT_RB][128];
    const int split = blockIdx.x, n_splits = gridDim.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kvh = h / (H / KVH);
    const int m_first = b * q_len;
    const int pos0 = pos[m_first];
    const size_t pstride = (size_t)hd + 2;
    if (pos0 < 0) {                                // sequence skipped: empty partials
        for (int idx = threadIdx.x; idx < q_len; idx += 256) {
            float* dst = part + ((((size_t)(m_first + idx)) * H + h) * n_splits + split) * pstride;
            dst[0] = -INFINITY; dst[1] = 0.f;
        }
        return;
    }
    const int n_keys = pos0 + q_len;
    const int tiles = (n_keys + 63) / 64;
    const int tiles_per_split = (tiles + n_splits - 1) / n_splits;
    const int t_begin = split * tiles_per_split;
    const int t_end = min(tiles, t_begin + tiles_per_split);
    const T* kb = k_cache + ((size_t)b * KVH + kvh) * (size_t)max_len * hd;
    const T* vb = v_cache + ((size_t)b * KVH + kvh) * (size_t)max_len * hd;
    const int d0 = lane, d1 = lane + 64;

    for (int r0 = 0; r0 < q_len; r0 += ATT_RB) {
        const int nr = min(ATT_RB, q_len - r0);
        __syncthreads();
        for (int idx = threadIdx.x; idx < ATT_RB * hd; idx += 256) {
            const int r = idx / hd, d = idx % hd;
            qs[r][d] = (r < nr) ? to_f(q[((size_t)(m_first + r0 + r) * H + h) * hd + d]) * scale : 0.f;
        }
        __syncthreads();
        float mrow[ATT_RB], lrow[ATT_RB], o0[ATT_RB], o1[ATT_RB];
#pragma unroll
        for (int r = 0; r < ATT_RB; ++r) { mrow[r] = -INFINITY; lrow[r] = 0.f; o0[r] = 0.f; o1[r] = 0.f; }

        for (int t = t_begin + wave; t < t_end; t += 4) {
            const int key = t * 64 + lane;
            const bool kvalid = key < n_keys;
            // ---- scores: lane = key ----
            float s[ATT_RB];
#pragma unroll
            for (int r = 0; r < ATT_RB; ++r) s[r] = 0.f;
            if (kvalid) {
                const T* krow = kb + (size_t)key * hd;
                for (int d = 0; d < hd; d += 8) {
                    float kv[8];
                    load8<T>(krow + d, kv);
#pragma unroll
                    for (int r = 0; r < ATT_RB; ++r) {
                        const float4 qa = *reinterpret_cast<const float4*>(&qs[r][d]);
                        const float4 qb = *reinterpret_cast<const float4*>(&qs[r][d + 4]);
                        s[r] += qa.x * kv[0] + qa.y * kv[1] + qa.z * kv[2] + qa.w * kv[3] +
                                qb.x * kv[4] + qb.y * kv[5] + qb.z * kv[6] + qb.w * kv[7];
                    }
                }
            }
            float alpha[ATT_RB];
#pragma unroll
            for (int r = 0; r < ATT_RB; ++r) {
                const bool vis = kvalid && r < nr && key <= pos0 + r0 + r;      // causal
                const float sv = vis ? s[r] : -INFINITY;
                const float mn = fmaxf(mrow[r], wmax(sv));
                const float pr = (mn == -INFINITY) ? 0.f : __expf(sv - mn);
                alpha[r] = (mn == -INFINITY) ? 1.f : __expf(mrow[r] - mn);
                lrow[r] = lrow[r] * alpha[r] + pr;                              // per-lane partial sum
                mrow[r] = mn;
                ps[wave][r][lane] = pr;
            }
            // ---- values: lane = head-dim element ----
#pragma unroll
            for (int r = 0; r < ATT_RB; ++r) { o0[r] *= alpha[r]; o1[r] *= alpha[r]; }
            const int kmax = min(64, n_keys - t * 64);
            for (int kk = 0; kk < kmax; kk += 4) {
                float v0[4], v1[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool okk = kk + u < kmax;
                    const T* vrow = vb + (size_t)(t * 64 + kk + u) * hd;
                    v0[u] = (okk && d0 < hd) ? to_f(vrow[d0]) : 0.f;
                    v1[u] = (okk && d1 < hd) ? to_f(vrow[d1]) : 0.f;
                }
#pragma unroll
                for (int r = 0; r < ATT_RB; ++r) {
                    const float4 pp = *reinterpret_cast<const float4*>(&ps[wave][r][kk]);
                    o0[r] += pp.x * v0[0] + pp.y * v0[1] + pp.z * v0[2] + pp.w * v0[3];
                    o1[r] += pp.x * v1[0] + pp.y * v1[1] + pp.z * v1[2] + pp.w * v1[3];
                }
            }
        }
        // ---- combine the 4 wavefronts ----
#pragma unroll
        for (int r = 0; r < ATT_RB; ++r) {
            const float l = wsum(lrow[r]);
            if (lane == 0) { wm[wave][r] = mrow[r]; wl[wave][r] = l; }
            wo[wave][r][d0] = o0[r];
            wo[wave][r][d1] = o1[r];
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < nr * hd; idx += 256) {
            const int r = idx / hd, d = idx % hd;
            const float mm = fmaxf(fmaxf(wm[0][r], wm[1][r]), fmaxf(wm[2][r], wm[3][r]));
            float o = 0.f, l = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = (wm[w][r] == -INFINITY) ? 0.f : __expf(wm[w][r] - mm);
                o += wo[w][r][d] * f;
                l += wl[w][r] * f;
            }
            float* dst = part + ((((size_t)(m_first + r0 + r)) * H + h) * n_splits + split) * pstride;
            dst[2 + d] = o;
            if (d == 0) { dst[0] = mm; dst[1] = l; }
        }
    }
}

// grid (M*H), threads hd: combine the splits, normalise, store in the storage dtype.
template <typename T>
__global__ void attn_merge_kernel(const float* __restrict__ part, int n_splits, int hd, T* __restrict__ out) {
    const size_t mh = blockIdx.x;
    const int d = threadIdx.x;
    const size_t pstride = (size_t)hd + 2;
    const float* base = part + mh * n_splits * pstride;
    float mm = -INFINITY;
    for (int s = 0; s < n_splits; ++s) mm = fmaxf(mm, base[s * pstride]);
    float o = 0.f, l = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float ms = base[s * pstride];
        const float f = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
        l += base[s * pstride + 1] * f;
        o += base[s * pstride + 2 + d] * f;
    }
    out[mh * hd + d] = from_f<T>(l > 0.f ? o / l : 0.f);
}

// ---- launchers -----------------------------------------------------------------------------------
int launch_prep(const int32_t* q_tokens, int q_stride, const int32_t* kv_len, int kv_base, int B, int q_len,
                int max_len, int V, int hd, float rope_base, int32_t* pos, int32_t* tok, float2* rope,
                int32_t* status, hipStream_t s) {
    hipLaunchKernelGGL(prep_kernel, dim3(B), dim3(128), 0, s, q_tokens, q_stride, kv_len, kv_base, q_len, max_len, V,
                       hd / 2, rope_base, pos, tok, rope, status);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_embed(int dtype, const int32_t* tok, const void* embed, int M, int d, float* x, hipStream_t s) {
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((embed_kernel<uint16_t>), dim3(M), dim3(256), 0, s, tok, (const uint16_t*)embed, d, x);
    else
        hipLaunchKernelGGL((embed_kernel<float>), dim3(M), dim3(256), 0, s, tok, (const float*)embed, d, x);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_rmsnorm(int dtype, const float* x, const float* gain, int d, float eps, int n_seq, int rows_in,
                   int rows_out, void* out, hipStream_t s) {
    const int rows = n_seq * rows_out;
    if (rows <= 0) return BS_OK;
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((rmsnorm_kernel<uint16_t>), dim3(rows), dim3(256), 0, s, x, gain, d, eps, rows_in, rows_out, (uint16_t*)out);
    else
        hipLaunchKernelGGL((rmsnorm_kernel<float>), dim3(rows), dim3(256), 0, s, x, gain, d, eps, rows_in, rows_out, (float*)out);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_rope_kv(int dtype, const float* qkv, const int32_t* pos, const float2* rope, int M, int q_len, int H,
                   int KVH, int hd, int max_len, void* q_out, void* k_cache, void* v_cache, hipStream_t s) {
    const dim3 grid(M, H + 2 * KVH), block(hd / 2);
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((rope_kv_kernel<uint16_t>), grid, block, 0, s, qkv, pos, rope, q_len, H, KVH, hd, max_len,
                           (uint16_t*)q_out, (uint16_t*)k_cache, (uint16_t*)v_cache);
    else
        hipLaunchKernelGGL((rope_kv_kernel<float>), grid, block, 0, s, qkv, pos, rope, q_len, H, KVH, hd, max_len,
                           (float*)q_out, (float*)k_cache, (float*)v_cache);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_attention(int dtype, const void* q, const void* k_cache, const void* v_cache, const int32_t* pos, int B,
                     int q_len, int H, int KVH, int hd, int max_len, int n_splits, float* part, void* out,
                     hipStream_t s) {
    const float scale = 1.0f / sqrtf((float)hd);
    const dim3 grid(n_splits, H, B), block(256);
    if (dtype == BS_BF16) {
        hipLaunchKernelGGL((attn_kernel<uint16_t>), grid, block, 0, s, (const uint16_t*)q, (const uint16_t*)k_cache,
                           (const uint16_t*)v_cache, pos, q_len, H, KVH, hd, max_len, scale, part);
        BS_LAUNCH_CHECK();
        hipLaunchKernelGGL((attn_merge_kernel<uint16_t>), dim3(B * q_len * H), dim3(hd), 0, s, part, n_splits, hd, (uint16_t*)out);
    } else {
        hipLaunchKernelGGL((attn_kernel<float>), grid, block, 0, s, (const float*)q, (const float*)k_cache,
                           (const float*)v_cache, pos, q_len, H, KVH, hd, max_len, scale, part);
        BS_LAUNCH_CHECK();
        hipLaunchKernelGGL((attn_merge_kernel<float>), dim3(B * q_len * H), dim3(hd), 0, s, part, n_splits, hd, (float*)out);
    }
    BS_LAUNCH_CHECK();
    return BS_OK;
}

}  // namespace bs
