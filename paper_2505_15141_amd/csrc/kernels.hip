// Device kernels of the transformer forward used by the verification pass (App. A: the target model
// scores all gamma+1 positions in one pass) and by the draft model's steps.
//
//   prep        positions, clamped tokens, RoPE cos/sin table, overflow status
//   embed       token embedding -> fp32 residual stream
//   rmsnorm     completes the fp32 residual from pending split-K partials, normalises it
//   gemm        y = x W^T: bf16 weights streamed once from HBM through MFMA 16x16x32 tiles (the
//               contraction is skinny: M = B*(gamma+1) rows, so it is bound by weight bandwidth),
//               split-K partials out; a many-row variant for prompt chunks and batches (activation
//               stages memory -> LDS directly, 256 x 256 tiles); fp32 variant for the fp32 plumbing
//               configuration
//   resid_sum   bf16 models: completes the residual, writes the planes of gain .* x and partial sums
//               of squares (the RMS scale is applied behind the projection)
//   gemm_dec    the same contraction for one or two rows (draft steps) with the layer's small kernels
//               folded into its epilogues (residual, RoPE + cache write, SwiGLU; RMSNorm by linearity)
//   swiglu      sums gate/up partials, applies silu(g)*u
//   rope_kv     sums q/k/v partials, rotates q and k, writes k/v into the cache
//   attention   q_len causal query rows per head against the contiguous KV cache, split along the
//               keys with online softmax; merge kernel combines the splits
#include <math.h>
#include <mutex>
#include <vector>
#include <hip/hip_ext.h>
#include "common.h"
#include "kernels.h"
#include "devutil.h"

namespace bs {

// ---- prep ---------------------------------------------------------------------------------------
// One workgroup per sequence.  pos[m] = kv_len[b] + kv_base + j, or -1 for a sequence that would run
// past max_len (then nothing of it is written anywhere).  tok[m] = token clamped into [0, V).
__global__ void prep_kernel(const int32_t* __restrict__ q_tokens, int q_stride, const int32_t* __restrict__ kv_len,
                            int kv_base, int q_len, int max_len, int V, int half_hd, float rope_base,
                            int32_t* __restrict__ pos, int32_t* __restrict__ tok, float2* __restrict__ rope,
                            int32_t* __restrict__ status, int B, uint4* __restrict__ clear, size_t clear16) {
    if ((int)blockIdx.x >= B) {                       // the blocks behind the sequences zero the exchange cells
        const size_t nb = gridDim.x - B;
        for (size_t i = (size_t)(blockIdx.x - B) * blockDim.x + threadIdx.x; i < clear16; i += nb * blockDim.x)
            clear[i] = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
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

// ---- activation format ---------------------------------------------------------------------------
// fp32 models keep activations as float [M, K].  bf16 models keep them as TWO bf16 planes hi, lo with
// hi = bf16(v), lo = bf16(v - hi): the MFMA GEMM multiplies the weight tile with both planes, so the
// activations enter the contraction with ~16 significant bits while the weights stream as bf16.  The
// matrix cores have a 20x surplus over the weight bandwidth at these row counts, so the second plane is free.
template <typename T> struct Act;
template <> struct Act<float> {
    static __device__ __forceinline__ void store(void* base, size_t plane, size_t idx, float v) {
        reinterpret_cast<float*>(base)[idx] = v;
    }
};
template <> struct Act<uint16_t> {
    static __device__ __forceinline__ void store(void* base, size_t plane, size_t idx, float v) {
        const uint16_t hi = from_f<uint16_t>(v);
        const uint16_t lo = from_f<uint16_t>(v - to_f(hi));
        reinterpret_cast<uint16_t*>(base)[idx] = hi;
        reinterpret_cast<uint16_t*>(base)[plane + idx] = lo;
    }
};

// Embedding for the fused small-batch schedule: x (fp32), the planes of gain .* x (the next projection's
// input; its epilogue applies the row's RMS scale, the projection being linear) and the row's sum of squares.
__global__ __launch_bounds__(256) void embed_dec_kernel(const int32_t* __restrict__ tok, const uint16_t* __restrict__ embed,
                                                        const float* __restrict__ gain, int d, float* __restrict__ x,
                                                        uint16_t* __restrict__ planes, size_t plane, float* __restrict__ ssq) {
    __shared__ float red[4];
    const int m = blockIdx.x;
    const uint16_t* row = embed + (size_t)tok[m] * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
        const float v = to_f(row[i]);
        x[(size_t)m * d + i] = v;
        Act<uint16_t>::store(planes, plane, (size_t)m * d + i, v * gain[i]);
        ss += v * v;
    }
    ss = wsum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ssq[m] = red[0] + red[1] + red[2] + red[3];
}

// four consecutive activations (index a multiple of 4) as two 8-byte stores, one per plane
__device__ __forceinline__ void store_planes4(uint16_t* base, size_t plane, size_t idx, float v0, float v1, float v2, float v3) {
    const uint16_t h0 = from_f<uint16_t>(v0), h1 = from_f<uint16_t>(v1), h2 = from_f<uint16_t>(v2), h3 = from_f<uint16_t>(v3);
    const uint16_t l0 = from_f<uint16_t>(v0 - to_f(h0)), l1 = from_f<uint16_t>(v1 - to_f(h1));
    const uint16_t l2 = from_f<uint16_t>(v2 - to_f(h2)), l3 = from_f<uint16_t>(v3 - to_f(h3));
    *reinterpret_cast<uint2*>(base + idx) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
    *reinterpret_cast<uint2*>(base + plane + idx) = make_uint2((uint32_t)l0 | ((uint32_t)l1 << 16), (uint32_t)l2 | ((uint32_t)l3 << 16));
}

// Activation planes for the whole-K projections of up to 16 rows (gemm_rows_kernel): [K/32][16 rows][32 columns], so that
// the B operand of one k step (16 rows x 64 bytes) is one contiguous kilobyte like a weight tile, instead of 16 pieces
// of 16 different cache lines.  A plane is 16*K elements whatever the row count; rows >= M are neither written nor read.
__device__ __forceinline__ size_t xt_index(int m, int k) { return (size_t)(k >> 5) * 512 + m * 32 + (k & 31); }

// ---- RMSNorm (+ pending split-K partials of the previous projection) -----------------------------
// out row r takes input row src = (r / rows_out) * rows_in + (rows_in - rows_out) + r % rows_out
// (rows_out = rows_in: identity; rows_out < rows_in: the trailing rows of every sequence).
// If pend != null the residual row is first completed: x[src] += sum_s pend[s][src][:], and written back.
template <typename T>
__global__ __launch_bounds__(1024) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ pend, int pend_ks,
                                                       size_t pend_stride, const float* __restrict__ gain, int d,
                                                       float eps, int rows_in, int rows_out, size_t plane,
                                                       void* __restrict__ out) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    const int src = (r / rows_out) * rows_in + (rows_in - rows_out) + r % rows_out;
    float* row = x + (size_t)src * d;
    const float* prow = pend ? pend + (size_t)src * d : nullptr;
    float ss = 0.f;
    // d % 8 == 0 (host check): float4 granules; the split-K partials are independent loads
    for (int i = threadIdx.x * 4; i < d; i += 4096) {
        float4 v = *reinterpret_cast<const float4*>(row + i);
        if (prow) {
            for (int s0 = 0; s0 < pend_ks; s0 += 4) {
                float4 p[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    p[u] = (s0 + u < pend_ks) ? *reinterpret_cast<const float4*>(prow + (size_t)(s0 + u) * pend_stride + i)
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < 4; ++u) { v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w; }
            }
            *reinterpret_cast<float4*>(row + i) = v;
        }
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wsum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x * 4; i < d; i += 4096) {
        const float4 v = *reinterpret_cast<const float4*>(row + i);        // own earlier write, or the input
        const float4 g = *reinterpret_cast<const float4*>(gain + i);
        Act<T>::store(out, plane, (size_t)r * d + i, v.x * scale * g.x);
        Act<T>::store(out, plane, (size_t)r * d + i + 1, v.y * scale * g.y);
        Act<T>::store(out, plane, (size_t)r * d + i + 2, v.z * scale * g.z);
        Act<T>::store(out, plane, (size_t)r * d + i + 3, v.w * scale * g.w);
    }
}

// ---- residual completion for bf16 models (the 16-row and many-row schedules) ---------------------------
// RMSNorm commutes with the projection that follows it (norm(x) W^T = r * ((gain .* x) W^T), r per row), so the
// row-wide reduction does not have to finish before the projection starts: this kernel only completes the residual
// (x += sum of the pending split-K partials), writes the planes of gain .* x and ONE partial sum of squares per
// 1024-column chunk; the projection's consumer (rope_kv, swiglu) multiplies by r.  grid (rows, ceil(d/1024)):
// every row is spread over several compute units instead of one.
__global__ __launch_bounds__(256) void resid_sum_kernel(float* __restrict__ x, const float* __restrict__ pend, int pend_ks,
                                                        size_t pend_stride, const float* __restrict__ gain, int d, size_t plane,
                                                        uint16_t* __restrict__ out, float* __restrict__ ssq, int tiled) {
    __shared__ float red[4];
    const int r = blockIdx.x, chunk = blockIdx.y, nchunks = gridDim.y;
    const int i = chunk * 1024 + threadIdx.x * 4;                 // d % 8 == 0 (host check): whole float4 granules
    float ss = 0.f;
    if (i < d) {
        float* row = x + (size_t)r * d + i;
        float4 v = *reinterpret_cast<const float4*>(row);
        if (pend) {
            const float* prow = pend + (size_t)r * d + i;
            for (int s0 = 0; s0 < pend_ks; s0 += 8) {
                float4 p[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    p[u] = *reinterpret_cast<const float4*>(prow + (size_t)min(s0 + u, pend_ks - 1) * pend_stride);
                    if (s0 + u >= pend_ks) p[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) { v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w; }
            }
            *reinterpret_cast<float4*>(row) = v;
        }
        ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        const float4 g = *reinterpret_cast<const float4*>(gain + i);
        store_planes4(out, plane, tiled ? xt_index(r, i) : (size_t)r * d + i, v.x * g.x, v.y * g.y, v.z * g.z, v.w * g.w);
    }
    ss = wsum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ssq[(size_t)r * nchunks + chunk] = red[0] + red[1] + red[2] + red[3];
}

// r = rsqrt(mean square + eps) of row m from its per-chunk sums of squares (null: no scaling)
__device__ __forceinline__ float row_rscale(const float* __restrict__ ssq, int nchunks, int m, float inv_d, float eps) {
    if (!ssq) return 1.f;
    float tot = 0.f;
    for (int c = 0; c < nchunks; ++c) tot += ssq[(size_t)m * nchunks + c];
    return 1.0f / sqrtf(tot * inv_d + eps);
}

// ---- SwiGLU over split-K partials: act = silu(sum_s g) * sum_s u, columns [0,ff) gate, [ff,2ff) up ------
template <typename T>
__global__ void swiglu_kernel(const float* __restrict__ part, int ks, size_t ks_stride, int M, int ff, size_t plane,
                              void* __restrict__ out, const float* __restrict__ ssq, int nchunks, float inv_d, float eps) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * ff) return;
    const size_t m = idx / ff, j = idx % ff;
    float g = 0.f, u = 0.f;
    for (int s = 0; s < ks; ++s) {
        g += part[(size_t)s * ks_stride + m * 2 * ff + j];
        u += part[(size_t)s * ks_stride + m * 2 * ff + ff + j];
    }
    const float rs = row_rscale(ssq, nchunks, (int)m, inv_d, eps);     // the input rows' RMS scale, if it was deferred
    g *= rs; u *= rs;
    Act<T>::store(out, plane, idx, g / (1.0f + __expf(-g)) * u);
}

// ---- GEMM, bf16 weights streamed through MFMA -------------------------------------------------------
// part[ks][m][n] = sum over the K range of split ks of x[m][k] * W[n][k].
// grid (ceil(N/64), KS), 4 wavefronts; wavefront w owns weight rows n0+16w .. n0+16w+15 (MFMA A operand:
// lane = (row l%16, k-slot l/16), one 16-byte load per 32-wide k slice, straight from HBM into registers,
// a whole stage of KC columns in flight per wavefront plus the next stage prefetched).  The activation
// slice [M, KC] of both planes is staged once per workgroup in LDS (rows padded by 16 bytes so that the
// 16 rows read by one ds_read_b128 phase fall into distinct banks) and shared by the four wavefronts.
// Each wavefront owns its output rows, so no cross-wavefront reduction is needed; split-K partials are
// summed by the consumer kernel.  Three kernels by row count: gemm_bf16_m16_kernel (up to 16 rows: pure weight
// streaming; the layers of a wide model take gemm_rows_kernel instead), this one with two row tiles (17..32 rows, and the
// fallback when K is not a multiple of 32), gemm_bf16_big_kernel from 33 rows on (measured faster from there).

// Weight layouts.  Row-major [N][K], or TILED: the matrix is cut into 64-row x 32-column blocks stored
// [N/64][K/32][4][64][8]: inside a block the four 16-row MFMA A tiles follow each other, and inside a tile the
// eight values of lane (row r, k-slot q) sit at lane index r + 16q.  One k step of a wavefront is then one
// contiguous kilobyte and the four wavefronts of a workgroup read 4 KiB runs, which is what HBM serves fastest
// (measured 3.6 -> 4.6 TB/s over the 7B layer shapes against 64-byte pieces 8 KiB apart).
// wlane_ptr: where lane (row local%16, k-slot lq) finds its chunk of k step 0; WSTEP: elements between k steps.
template <bool TILED> struct WSTEP { static constexpr int v = TILED ? 2048 : 32; };
template <bool TILED>
__device__ __forceinline__ const uint16_t* wlane_ptr(const uint16_t* w, int local, int K, int lq) {
    if (TILED) return w + (size_t)(local >> 6) * 64 * K + ((local >> 4) & 3) * 512 + ((local & 15) + 16 * lq) * 8;
    return w + (size_t)local * K + lq * 8;
}

// Column offset of a k slice that starts at k, clamped into the row for the lane whose pointer already sits at k-slot lq
// (tiled: K % 32 == 0, whole slices; row-major: K % 8 == 0, the lane's 8-column chunk must end inside the row).
template <bool TILED>
__device__ __forceinline__ int wclamp(int k, int K, int lq) {
    if (TILED) return min(k, K - 32);
    return max(min(k, K - 8 - lq * 8), -lq * 8);
}

// dst (tiled, rows padded to a multiple of 64 with zeros) <- src (row-major [N][K]); one 16-byte chunk per lane.
__global__ void pack_weights_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int N, int K) {
    const size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_block = (size_t)(K / 32) * 256;                  // chunks per 64-row block
    const size_t nblocks = (size_t)((N + 63) / 64);
    if (c >= nblocks * per_block) return;
    const int nb = (int)(c / per_block);
    const size_t rem = c % per_block;
    const int step = (int)(rem / 256), in = (int)(rem % 256);
    const int t = in >> 6, lane = in & 63;
    const int n = nb * 64 + t * 16 + (lane & 15), k = step * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = ldg16(src + (size_t)n * K + k);
    *reinterpret_cast<uint4*>(dst + c * 8) = v;
}

template <int MT, int NT, int KC, bool TILED>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs a) {
    constexpr int ROW = KC + 8;                       // padded LDS row (bf16 elements)
    constexpr int NSL = KC / 32;                      // k slices per stage
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][MT * 16][ROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int n0 = blockIdx.x * (64 * NT) + wave * (16 * NT);    // this wavefront: NT tiles of 16 weight rows
    const uint16_t* wrow[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        int n = n0 + u * 16 + li;
        if (n >= a.N) n = a.N - 1;
        int seg = 0, local = n;
        if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
        wrow[u] = wlane_ptr<TILED>(reinterpret_cast<const uint16_t*>(a.w[seg]), local, a.K, lq);
    }
    const uint16_t* xh = reinterpret_cast<const uint16_t*>(a.x);
    const uint16_t* xl = xh + a.x_plane;
    // stages of this split
    const int nstages = (a.K + KC - 1) / KC;
    const int ks = blockIdx.y, KS = gridDim.y;
    const int st_begin = (int)((long long)nstages * ks / KS), st_end = (int)((long long)nstages * (ks + 1) / KS);

    f32x4 acc[NT][MT];
#pragma unroll
    for (int u = 0; u < NT; ++u)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 wcur[NT][NSL], wnext[NT][NSL];
    auto load_stage = [&](int st, uint4 (&dst)[NT][NSL]) {
        const int kb = st * KC;                       // wrow already points at this lane's k-slot
#pragma unroll
        for (int u = 0; u < NT; ++u)
#pragma unroll
            for (int j = 0; j < NSL; ++j) {
                // unconditional and clamped (a select on the loaded value would make the wavefront wait for it right here):
                // columns past K re-read the row's last chunk and meet zero activations, stages past the end are never used
                const int k = wclamp<TILED>(kb + j * 32, a.K, lq);
                dst[u][j] = ldg16(wrow[u] + (size_t)k * (WSTEP<TILED>::v / 32));
            }
    };
    // Activation slice of a stage: 16-byte chunks, rows >= M and columns >= K are zero.  It is requested into registers
    // one stage ahead (behind the weight prefetch) and written to LDS after the MFMAs of the current stage, so the trip
    // to memory hides behind them.
    constexpr int CHUNKS = 2 * MT * 16 * (KC / 8);
    constexpr int XPT = (CHUNKS + 255) / 256;         // chunks per lane
    uint4 xr[XPT];
    auto load_x = [&](int st) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int c = threadIdx.x + i * 256;
            const int plane = c / (MT * 16 * (KC / 8));
            const int rem = c % (MT * 16 * (KC / 8));
            const int m = rem / (KC / 8), kc = (rem % (KC / 8)) * 8;
            const int k = st * KC + kc;
            const bool ok = c < CHUNKS && st < st_end && m < a.M && k < a.K;
            const uint4 v = ldg16((plane ? xl : xh) + (ok ? (size_t)m * a.K + k : 0));       // always a valid address
            xr[i] = ok ? v : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_x = [&]() {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int c = threadIdx.x + i * 256;
            if (c < CHUNKS) {
                const int plane = c / (MT * 16 * (KC / 8));
                const int rem = c % (MT * 16 * (KC / 8));
                *reinterpret_cast<uint4*>(&xs[plane][rem / (KC / 8)][(rem % (KC / 8)) * 8]) = xr[i];
            }
        }
    };
    load_stage(st_begin, wcur);
    load_x(st_begin);
    store_x();
    __syncthreads();
    for (int st = st_begin; st < st_end; ++st) {
        load_stage(st + 1, wnext);                    // prefetch (all zero past the end)
        load_x(st + 1);
#pragma unroll
        for (int j = 0; j < NSL; ++j) {
#pragma unroll
            for (int t = 0; t < MT; ++t) {            // one pair of activation operands serves the NT weight tiles
                const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xs[0][t * 16 + li][j * 32 + lq * 8]));
                const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xs[1][t * 16 + li][j * 32 + lq * 8]));
#pragma unroll
                for (int u = 0; u < NT; ++u) {
                    const bf16x8 A = __builtin_bit_cast(bf16x8, wcur[u][j]);
                    acc[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, bh, acc[u][t], 0, 0, 0);
                    acc[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, bl, acc[u][t], 0, 0, 0);
                }
            }
        }
        __syncthreads();                              // every wavefront is done reading this stage's slice
        store_x();
        __syncthreads();
#pragma unroll
        for (int u = 0; u < NT; ++u)
#pragma unroll
            for (int j = 0; j < NSL; ++j) wcur[u][j] = wnext[u][j];
    }
    // D[n = n0 + 16u + 4*lq + e][m = 16t + li]: four consecutive n per lane -> one 16-byte store
    float* out = reinterpret_cast<float*>(a.out) + (size_t)ks * a.ks_stride;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const int nb = n0 + u * 16 + 4 * lq;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = t * 16 + li;
            if (m >= a.M) continue;
            float* o = out + (size_t)m * a.ldo + nb;
            if (nb + 3 < a.N && (reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                *reinterpret_cast<float4*>(o) = make_float4(acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (nb + e < a.N) o[e] = acc[u][t][e];
            }
        }
    }
}

// ---- GEMM for 33 activation rows and more (prompt processing, verification of a batch) -----------------
// From about 150 rows on the projections are bound by the matrix cores, not by the weight stream (two MFMAs per
// weight tile and activation tile because of the two planes), and what then limits a workgroup is how many
// operand bytes it pulls out of LDS per MFMA and how far ahead its operands are requested.  Sized for that
// (and, with fewer row tiles, still ahead of the kernel above from 33 rows on: 140 against 195 us for the four
// projections of a 7B layer at 80 rows):
//   * 8 wavefronts as 4 (weight rows) x 2 (activation rows): a wavefront multiplies 64 weight rows (4 tiles, in
//     registers) with half of the activation tiles, so an activation tile read from LDS feeds 8 MFMAs;
//   * stages of 32 columns; the activation slice of a stage goes memory -> LDS directly (16 bytes per lane, the
//     lanes of a wavefront fill one contiguous KB = one 16-row tile of one plane, chunks placed so that reading
//     the MFMA B operand back is one conflict-free 16-byte read per lane) into a ring of 4 buffers, three stages ahead;
//   * the weight tiles of a stage sit in a register ring of 3 stages.
// Every load of a stage is issued unconditionally and in the same order by every wavefront, so the wait before a
// stage is a count: all but the loads of the newest stage (a stage is waited for one stage early, so that its first
// tile can be read from LDS before the barrier).  Rows past M re-read row M-1 (their results
// are not stored), stages past the end re-read the last stage into a buffer nobody reads.
// MT (even) is the number of 16-row activation tiles: 144 rows (a batch of 16 sequences being verified) take 10
// tiles, not 16, so the matrix cores do not multiply rows that do not exist.
constexpr int BIG_WAVES = 8, BIG_STAGES = 4;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// two 16-byte LDS reads at addr + OA and addr + OB (bytes, below 64 KiB); the data is there after lds_wait
template <int OA, int OB>
__device__ __forceinline__ void lds_read_pair(u32x4& a, u32x4& b, uint32_t addr) {
    static_assert(OA >= 0 && OA < 65536 && OB >= 0 && OB < 65536, "16-bit instruction offset");
    asm volatile("ds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4" : "=&v"(a), "=&v"(b) : "v"(addr), "n"(OA), "n"(OB) : "memory");
}
__device__ __forceinline__ void lds_wait(u32x4& a, u32x4& b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)); }

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (the other counters unconstrained)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

template <int MT, bool TILED>
__global__ __launch_bounds__(64 * BIG_WAVES) void gemm_bf16_big_kernel(GemmArgs a) {
    static_assert(MT % 2 == 0 && MT >= 2 && MT <= 16, "row tiles split evenly over the two wavefront rows");
    constexpr int MTW = MT / 2;                       // activation tiles per wavefront
    constexpr int NF = (2 * MT + BIG_WAVES - 1) / BIG_WAVES;      // 1 KB pieces of a stage each wavefront fetches
    constexpr int SLOT = NF + 4;                      // vector-memory operations per stage and wavefront
    static_assert(2 * SLOT < 64, "the wait count has six bits");
    __shared__ __attribute__((aligned(16))) uint16_t xs[BIG_STAGES][2 * MT][512];     // [buffer][plane * MT + tile][16 rows x 32 columns]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int wn = wave & 3, wm = wave >> 2;
    // Work item = (split of K, tile of 256 weight rows, block of 256 activation rows), in that order of significance.
    // Workgroups go round the 8 dies (linear id modulo 8), each die with its own L2: die x takes the x-th eighth of the
    // item list, so that it works on one or two K ranges only -- it reads just that slice of the activations (which all
    // its tiles share) and each of its weight tiles once for all row blocks.  With the tiles dealt round the dies
    // instead, every die read ALL activations: 450 MB from memory for the 135 MB of the 7B down projection at 1024 rows.
    const int n_mb = (a.M + 255) / 256, n_tiles = (a.N + 255) / 256;
    const int n_tiles_pad = (n_tiles + 7) & ~7, KS = gridDim.y;
    const int lin = blockIdx.x + gridDim.x * blockIdx.y;           // gridDim.x = n_tiles_pad * n_mb
    const int per_die = (n_tiles_pad * n_mb * KS) >> 3;
    const int item = (lin & 7) * per_die + (lin >> 3);
    const int ks = item / (n_tiles_pad * n_mb), rem = item - ks * (n_tiles_pad * n_mb);
    const int tile = rem / n_mb, m_off = (rem - tile * n_mb) * 256;
    if (tile >= n_tiles) return;                                   // the grid is padded to whole groups of 8 tiles
    const int M = min(a.M - m_off, 256);
    const int n0 = tile * 256 + wn * 64;
    const uint16_t* wrow[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        int n = n0 + u * 16 + li;
        if (n >= a.N) n = a.N - 1;
        int seg = 0, local = n;
        if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
        wrow[u] = wlane_ptr<TILED>(reinterpret_cast<const uint16_t*>(a.w[seg]), local, a.K, lq);
    }
    const uint16_t* xh = reinterpret_cast<const uint16_t*>(a.x) + (size_t)m_off * a.K;
    const int nstages = a.K / 32;                     // K % 32 == 0 (host check)
    const int st_begin = (int)((long long)nstages * ks / KS), st_end = (int)((long long)nstages * (ks + 1) / KS);
    const int st_last = max(st_end - 1, st_begin);
    // this wavefront's pieces of a stage: piece p = plane * MT + tile.  The transfer puts lane l's 16 bytes at offset
    // 16 l of the piece.  Four consecutive lanes fetch the four 16-byte chunks of one row (one 64-byte run: the
    // address unit works on such lane quads), rotated by row / 2, so that row r's chunk c sits at slot
    // 4 r + ((c + r / 2) & 3): LDS serves 8 lanes x 16 bytes per cycle, and the 8 lanes that read one k-slot of 8
    // consecutive rows then hit 8 different 16-byte bank groups (measured: no conflicts; rotating by row / 4 gave 2-way).
    const uint16_t* fsrc[NF];
    int fpiece[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int p = min(wave + BIG_WAVES * f, 2 * MT - 1);      // a surplus fetch repeats the last piece (same bytes)
        const int plane = p / MT, rt = p - plane * MT;
        fpiece[f] = p;
        fsrc[f] = xh + (size_t)plane * a.x_plane + (size_t)min(rt * 16 + (lane >> 2), M - 1) * a.K + (((lane & 3) - (lane >> 3)) & 3) * 8;
    }
    auto fill = [&](int st, int buf) {
        const int s = min(st, st_last);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            __builtin_amdgcn_global_load_lds((global_void_ptr)(fsrc[f] + (size_t)s * 32), (lds_void_ptr)&xs[buf][fpiece[f]][0], 16, 0, 0);
    };
    auto wload = [&](int st, uint4 (&dst)[4]) {
        const int s = min(st, st_last);
#pragma unroll
        for (int u = 0; u < 4; ++u) dst[u] = ldg16(wrow[u] + (size_t)s * WSTEP<TILED>::v);
    };
    f32x4 acc[4][MTW];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int t = 0; t < MTW; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint4 w0[4], w1[4], w2[4];
    fill(st_begin, 0);     wload(st_begin, w0);
    fill(st_begin + 1, 1); wload(st_begin + 1, w1);
    fill(st_begin + 2, 2); wload(st_begin + 2, w2);
    // "Everything but the newest stage has landed", then a bare barrier: for every wavefront's pieces, and every
    // wavefront is done reading the stage before.  __syncthreads() would add a release fence, which has to wait for ALL
    // transfers into LDS, the prefetched stages included.
    auto landed = [&]() {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(SLOT));
        __builtin_amdgcn_s_barrier();
    };
    // The activation tiles are read with explicit LDS instructions and explicit waits: an LDS load the compiler knows
    // about would be made to wait for EVERY transfer into LDS still in flight (it cannot tell the buffers apart).
    u32x4 bq[2][2];
    landed();                                                      // stages st_begin and st_begin + 1
    const int bslot = 4 * li + ((lq + (li >> 1)) & 3);              // where this lane's B operand (row li, k-slot lq) sits in a piece
    lds_read_pair<0, MT * 1024>(bq[0][0], bq[0][1], lds_addr(&xs[0][wm * MTW][bslot * 8]));
    // One stage.  On entry its first tile is already on its way into bq[0], and the next stage has landed as well, so
    // that stage's first tile is requested before this stage's last MFMAs: no LDS latency is exposed at the barrier.
    // The pieces of stage st+3 (into the buffer of stage st-1, which everybody has left) are requested between the MFMA groups.
    auto step = [&](int st, uint4 (&w)[4], bool prefetch) {
        const int buf = (st - st_begin) & (BIG_STAGES - 1);
        const uint32_t bh = lds_addr(&xs[buf][wm * MTW][bslot * 8]);                         // plane 0; plane 1 is MT KB further
        const uint32_t bh_next = lds_addr(&xs[(buf + 1) & (BIG_STAGES - 1)][wm * MTW][bslot * 8]);
        const int s3 = min(st + 3, st_last), buf3 = (buf + 3) & (BIG_STAGES - 1);
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            const int slot = t & 1;
            lds_wait(bq[slot][0], bq[slot][1]);
            lds_read_pair<0, MT * 1024>(bq[slot ^ 1][0], bq[slot ^ 1][1], t + 1 < MTW ? bh + (t + 1) * 1024 : bh_next);
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 Bh = __builtin_bit_cast(bf16x8, bq[slot][0]), Bl = __builtin_bit_cast(bf16x8, bq[slot][1]);
#pragma unroll
            for (int u = 0; u < 4; ++u)                            // the two MFMAs on one accumulator are kept apart
                acc[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), Bh, acc[u][t], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), Bl, acc[u][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (prefetch && t < NF)
                __builtin_amdgcn_global_load_lds((global_void_ptr)(fsrc[t] + (size_t)s3 * 32), (lds_void_ptr)&xs[buf3][fpiece[t]][0], 16, 0, 0);
        }
        static_assert(NF <= MTW, "one piece per MFMA group");
        if (prefetch) wload(st + 3, w);
        if (MTW & 1) {                                             // the next stage's first tile went to bq[1]: it is expected in bq[0]
            lds_wait(bq[1][0], bq[1][1]);
            bq[0][0] = bq[1][0]; bq[0][1] = bq[1][1];
        }
        landed();                                                  // stage st+2; and everybody is done with stage st
    };
    // Whole groups of three stages run without a branch, so that the compiler can count the loads in flight; the
    // one or two stages left over request nothing any more.
    int st = st_begin;
    for (; st + 3 <= st_end; st += 3) {
        step(st, w0, true);
        step(st + 1, w1, true);
        step(st + 2, w2, true);
    }
    if (st < st_end) {
        step(st, w0, false);
        if (st + 1 < st_end) step(st + 1, w1, false);
    }
    lds_wait(bq[0][0], bq[0][1]);                                  // the read ahead of the last stage is not used
    lds_wait(bq[1][0], bq[1][1]);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                      // no transfer into LDS is left in flight
    // Stored straight from the registers (a lane holds D[column 16u + 4 lq + e][row 16t + li]).  Routing the block through
    // LDS to write whole 256-byte rows was measured and changed nothing: what the output costs is its size -- every
    // split writes M x 256 floats per workgroup and the launch ends when they are in memory (7 us for 4 MB, 14 us for 64 MB).
    float* out = reinterpret_cast<float*>(a.out) + (size_t)ks * a.ks_stride + (size_t)m_off * a.ldo;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int nb = n0 + u * 16 + 4 * lq;
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            const int m = (wm * MTW + t) * 16 + li;
            if (m >= M) continue;
            float* o = out + (size_t)m * a.ldo + nb;
            if (nb + 3 < a.N && (reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                *reinterpret_cast<float4*>(o) = make_float4(acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (nb + e < a.N) o[e] = acc[u][t][e];
            }
        }
    }
}

// ---- GEMM for at most 16 activation rows (LM heads; the layers of models too narrow for gemm_rows_kernel) ----
// Same operand mapping as above, but the whole K range of the workgroup (at most M16_KMAX columns) is
// staged in LDS once, behind the first weight loads, and the loop over 32-wide k slices then runs without
// barriers: each wavefront keeps a ring of M16_DEPTH weight loads (16 rows x 64 bytes each) in flight and
// retires them in order against the in-order memory counter.
constexpr int M16_KMAX = 512;
constexpr int M16_DEPTH = 8;

template <int NT, bool TILED>
__global__ __launch_bounds__(256) void gemm_bf16_m16_kernel(GemmArgs a, int kper) {
    constexpr int ROW = M16_KMAX + 8;
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][16][ROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int n0 = blockIdx.x * (64 * NT) + wave * (16 * NT);      // this wavefront: NT tiles of 16 weight rows
    const int ks = blockIdx.y;
    const int k_lo = ks * kper, k_hi = min(a.K, k_lo + kper);       // this workgroup's columns
    const uint16_t* wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int n = n0 + t * 16 + li;
        if (n >= a.N) n = a.N - 1;
        int seg = 0, local = n;
        if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
        wrow[t] = wlane_ptr<TILED>(reinterpret_cast<const uint16_t*>(a.w[seg]), local, a.K, lq);
    }
    const uint16_t* xh = reinterpret_cast<const uint16_t*>(a.x);
    const uint16_t* xl = xh + a.x_plane;
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    // phases of at most M16_KMAX columns (one phase unless the caller asked for few splits)
    for (int k_begin = k_lo; k_begin < k_hi; k_begin += M16_KMAX) {
        const int k_end = min(k_hi, k_begin + M16_KMAX);
        const int nsl = (k_end - k_begin + 31) / 32;
        // Unconditional loads (a branch around a load would force the compiler to wait for every outstanding
        // load instead of counting them): slices past the end re-read the last valid 16-byte chunk of the row,
        // which meets zero activations in LDS.
        const int k_last = k_end - 8 - lq * 8;             // last valid chunk start for this lane's k-slot
        auto wload = [&](int t, int j) {
            if (TILED) return ldg16(wrow[t] + (size_t)min(k_begin + j * 32, k_end - 32) * 64);   // K % 32 == 0
            const int k = max(min(k_begin + j * 32, k_last), -lq * 8);   // wrow already points at column lq*8
            return ldg16(wrow[t] + k);
        };
        // Activation slice [16][k_begin..k_end) of both planes: requested first (L2 hits), the weight ring
        // right behind it, so that the LDS fill waits for the slice only (the memory counter retires in order).
        // 2 planes x 16 rows x 64 chunks of 16 bytes = 8 chunks per lane; rows >= M and the tail are zero.
        constexpr int XCH = 2 * 16 * (M16_KMAX / 8) / 256;      // fixed geometry: chunk c -> (plane, row, column) by shifts
        static_assert(M16_KMAX == 512, "chunk decoding below assumes 64 chunks per row");
        uint4 xv[XCH];
#pragma unroll
        for (int u = 0; u < XCH; ++u) {
            const int c = threadIdx.x + u * 256;
            const int plane = c >> 10, m = (c >> 6) & 15, kc = (c & 63) * 8;
            const bool ok = m < a.M && k_begin + kc < k_end;
            const uint16_t* src = (plane ? xl : xh) + (ok ? (size_t)m * a.K + k_begin + kc : 0);   // always a valid address
            xv[u] = ldg16(src);
            const uint32_t keep = ok ? 0xFFFFFFFFu : 0u;
            xv[u].x &= keep; xv[u].y &= keep; xv[u].z &= keep; xv[u].w &= keep;
        }
        uint4 w[NT][M16_DEPTH];
#pragma unroll
        for (int u = 0; u < M16_DEPTH; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) w[t][u] = wload(t, u);
        if (k_begin != k_lo) __syncthreads();              // the previous phase's LDS reads are done
#pragma unroll
        for (int u = 0; u < XCH; ++u) {
            const int c = threadIdx.x + u * 256;
            *reinterpret_cast<uint4*>(&xs[c >> 10][(c >> 6) & 15][(c & 63) * 8]) = xv[u];
        }
        __syncthreads();
        for (int j0 = 0; j0 < nsl; j0 += M16_DEPTH) {
#pragma unroll
            for (int u = 0; u < M16_DEPTH; ++u) {
                bf16x8 A[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    A[t] = __builtin_bit_cast(bf16x8, w[t][u]);
                    w[t][u] = wload(t, j0 + M16_DEPTH + u);
                }
                const int j = j0 + u;
                if (j < nsl) {
                    const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xs[0][li][j * 32 + lq * 8]));
                    const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xs[1][li][j * 32 + lq * 8]));
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[t], bh, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[t], bl, acc[t], 0, 0, 0);
                    }
                }
            }
        }
    }
    float* out = a.out + (size_t)ks * a.ks_stride;
    if (li < a.M) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int nb = n0 + t * 16 + 4 * lq;
            float* o = out + (size_t)li * a.ldo + nb;
            if (nb + 3 < a.N && (reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                *reinterpret_cast<float4*>(o) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (nb + e < a.N) o[e] = acc[t][e];
            }
        }
    }
}

// ---- fused projections for very few rows (draft steps) ----------------------------------------------
// With one or two activation rows every kernel of a layer is a few microseconds of latency, so the layer
// time is the number of kernels.  Here a workgroup owns 16 output columns over the WHOLE K range: its
// wavefronts split K, add their accumulators through LDS, and wavefront 0 finishes the columns in place:
//   EPI_RESID   x += y; planes of gain_next .* x and the 16-column sums of squares for the next RMSNorm
//   EPI_QKV     RMS scale of the input rows, RoPE on q and k, q out (fp32), k and v into the cache
//   EPI_SWIGLU  gate and up tiles of the same columns side by side: silu(r g) * (r u) as planes
// so a layer is 4 projections + attention + merge instead of 10 kernels.  RMSNorm commutes with the
// projection: norm(x) W^T = r * ((gain .* x) W^T), r = rsqrt(mean(x^2) + eps) per row, so the producer of x
// writes gain .* x and partial sums of squares, and the consumer of the projection multiplies by r.
// The activations come straight from L2 (MFMA B operand: lane = (row l%16, k-slot l/16)); that costs twice
// the weight bytes in L1 traffic at 16 rows, which is why this path is for a handful of rows only.
// Weights are in the tiled layout.

template <int EPI, int DEPTH, bool MERGE>
__global__ __launch_bounds__(512) void gemm_dec_kernel(DecArgs a) {
    __shared__ __attribute__((aligned(16))) float red[8][256];
    extern __shared__ __attribute__((aligned(16))) uint16_t xs[];     // [2 planes][M][K + 8]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int WS = EPI == EPI_SWIGLU ? W / 2 : W;                 // K splits per 16-column tile
    const int grp = wave / WS, split = wave - grp * WS;
    const int n0 = blockIdx.x * 16;
    const int c = n0 + 4 * lq;                                    // lane's four output columns (epilogue)
    const bool row_ok = li < a.M;
    const uint16_t* wmat;
    int local = n0 + li;
    if (EPI == EPI_SWIGLU) wmat = reinterpret_cast<const uint16_t*>(a.w[grp]);
    else {
        int seg = 0;
        if (a.w[1] && local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (a.w[2] && local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
        wmat = reinterpret_cast<const uint16_t*>(a.w[seg]);
    }
    // Everything the epilogue needs from memory is requested now, ahead of the operand streams, so that it has
    // arrived long before wavefront 0 gets there: the rows' sums of squares, the residual and gain (RESID),
    // position and rotation (QKV).
    float ssr[DEC_MAX_ROWS];                                      // this lane's share of each row's sum of squares
#pragma unroll
    for (int m = 0; m < DEC_MAX_ROWS; ++m) ssr[m] = 0.f;
    float4 x_old = make_float4(0.f, 0.f, 0.f, 0.f), g_next = make_float4(0.f, 0.f, 0.f, 0.f);
    float2 rc0 = make_float2(1.f, 0.f), rc1 = make_float2(1.f, 0.f);
    int p_row = -1;
    const int hd_mask = a.hd - 1;                                 // head_dim is 64 or 128
    if (wave == 0) {
        const int m = min(li, a.M - 1);
        if (EPI != EPI_RESID) {
#pragma unroll
            for (int mm = 0; mm < DEC_MAX_ROWS; ++mm) {
                if (mm >= a.M) break;
                for (int t = lane; t < a.ssq_tiles; t += 256) {       // independent loads, four per lane in flight
                    float v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int tt = t + 64 * u;
                        v[u] = a.ssq_in[(size_t)mm * a.ssq_tiles + min(tt, a.ssq_tiles - 1)];
                        if (tt >= a.ssq_tiles) v[u] = 0.f;
                    }
                    ssr[mm] += (v[0] + v[1]) + (v[2] + v[3]);
                }
            }
        }
        if (EPI == EPI_RESID) {
            x_old = *reinterpret_cast<const float4*>(a.x + (size_t)m * a.N + c);
            if (a.gain_next) g_next = *reinterpret_cast<const float4*>(a.gain_next + c);
        }
        if (EPI == EPI_QKV) {
            p_row = a.pos[m];
            const int hc = c & hd_mask;
            rc0 = a.rope[(size_t)m * (a.hd / 2) + hc / 2];
            rc1 = a.rope[(size_t)m * (a.hd / 2) + hc / 2 + 1];
        }
    }
    // ---- activations: both planes of all M rows, whole K, into LDS (a few KB at these row counts) ----
    // First round of 16-byte chunks is requested BEFORE the weight prologue and stored after it, so that the
    // wait for it (the memory counter retires in order) leaves the weight loads in flight.
    const int row_e = a.K + 8;                                    // padded row, elements
    const int kc8 = a.K / 8;                                      // 16-byte chunks per row
    const int kc0 = threadIdx.x < (unsigned)kc8 ? (int)threadIdx.x : 0;       // lanes past the row re-read chunk 0 (not stored)
    uint4 xv0[2 * DEC_MAX_ROWS];
    if (!MERGE) {
#pragma unroll
        for (int pr = 0; pr < 2 * DEC_MAX_ROWS; ++pr) {           // pr = plane * M + row, clamped to the last valid pair
            const int q = min(pr, 2 * a.M - 1);
            const int plane = q >= a.M ? 1 : 0, m = q - plane * a.M;
            xv0[pr] = ldg16(a.xh + (size_t)plane * a.x_plane + (size_t)m * a.K + kc0 * 8);
        }
    }
    const int steps = a.K / 32;
    const int ws_shift = __ffs(WS) - 1;                           // WS is 4 or 8
    const int s_begin = (split * steps) >> ws_shift, s_end = ((split + 1) * steps) >> ws_shift;
    const int n = s_end - s_begin;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const char* wb = reinterpret_cast<const char*>(wmat);
    // byte offsets (every matrix is below 4 GiB: host check); a k step is 4096 bytes of the tiled weights
    uint32_t woff = (uint32_t)(((size_t)(local >> 6) * 64 * a.K + ((local >> 4) & 3) * 512 + ((local & 15) + 16 * lq) * 8 +
                                (size_t)s_begin * 2048) * 2);
    uint4 rw[DEPTH];
    {
        const int nn = max(n, 1) - 1;                             // n == 0: the wavefront re-reads step 0 of its tile and ignores it
        const uint32_t w0 = n > 0 ? woff : (uint32_t)(((size_t)(local >> 6) * 64 * a.K + ((local >> 4) & 3) * 512 + ((local & 15) + 16 * lq) * 8) * 2);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) rw[u] = ldg16((const uint16_t*)(wb + w0 + min(u, nn) * 4096));   // clamped to the last step
    }
    if (!MERGE) {
#pragma unroll
        for (int pr = 0; pr < 2 * DEC_MAX_ROWS; ++pr)
            if (pr < 2 * a.M && threadIdx.x < (unsigned)kc8) *reinterpret_cast<uint4*>(&xs[pr * row_e + threadIdx.x * 8]) = xv0[pr];
        for (int pr = 0; pr < 2 * a.M; ++pr) {                    // rows longer than the workgroup (8 columns per lane): the rest
            const int plane = pr >= a.M ? 1 : 0, m = pr - plane * a.M;
            for (int kc = threadIdx.x + blockDim.x; kc < kc8; kc += blockDim.x)
                *reinterpret_cast<uint4*>(&xs[pr * row_e + kc * 8]) = ldg16(a.xh + (size_t)plane * a.x_plane + (size_t)m * a.K + kc * 8);
        }
    } else {
        // The activations are the attention output, still as per-split partials (o[hd], max, sum): each lane combines
        // the splits of eight head-dim elements (online over groups of 8 splits, all loads of a group in flight) and
        // writes both planes.  Every workgroup redoes this for the whole row: a few KB from L2, one kernel fewer.
        const size_t pstride = (size_t)a.hd + 4;
        const int hd_shift = __ffs(a.hd) - 1;
        for (int m = 0; m < a.M; ++m)
            for (int kc = threadIdx.x; kc < kc8; kc += blockDim.x) {
                const int col = kc * 8, h = col >> hd_shift, d0 = col & (a.hd - 1);
                const float* base = a.att_part + ((size_t)m * a.H + h) * a.att_splits * pstride;
                float mm = -INFINITY, lsum = 0.f, o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = 0.f;
                for (int s0 = 0; s0 < a.att_splits; s0 += 8) {
                    float4 oa[8], ob[8];
                    float2 ml[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float* ps = base + (size_t)min(s0 + u, a.att_splits - 1) * pstride;
                        oa[u] = *reinterpret_cast<const float4*>(ps + d0);
                        ob[u] = *reinterpret_cast<const float4*>(ps + d0 + 4);
                        ml[u] = *reinterpret_cast<const float2*>(ps + a.hd);
                        if (s0 + u >= a.att_splits) ml[u] = make_float2(-INFINITY, 0.f);
                    }
                    float gm = mm;
#pragma unroll
                    for (int u = 0; u < 8; ++u) gm = fmaxf(gm, ml[u].x);
                    if (gm == -INFINITY) continue;
                    const float keep = __expf(mm - gm);                  // 0 when nothing was accumulated yet
                    lsum *= keep;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] *= keep;
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float f = (ml[u].x == -INFINITY) ? 0.f : __expf(ml[u].x - gm);
                        if (f == 0.f) continue;                          // an empty split's o[] was never written
                        lsum += ml[u].y * f;
                        o[0] += oa[u].x * f; o[1] += oa[u].y * f; o[2] += oa[u].z * f; o[3] += oa[u].w * f;
                        o[4] += ob[u].x * f; o[5] += ob[u].y * f; o[6] += ob[u].z * f; o[7] += ob[u].w * f;
                    }
                    mm = gm;
                }
                const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
                uint32_t hw[4], lw[4];
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float v0 = o[e] * inv, v1 = o[e + 1] * inv;
                    const uint16_t h0 = from_f<uint16_t>(v0), h1 = from_f<uint16_t>(v1);
                    hw[e / 2] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                    lw[e / 2] = (uint32_t)from_f<uint16_t>(v0 - to_f(h0)) | ((uint32_t)from_f<uint16_t>(v1 - to_f(h1)) << 16);
                }
                *reinterpret_cast<uint4*>(&xs[(size_t)m * row_e + col]) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                *reinterpret_cast<uint4*>(&xs[(size_t)(a.M + m) * row_e + col]) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
            }
    }
    __syncthreads();                                              // activations are in LDS
    if (n > 0) {
        // MFMA B operand: lane (row l%16, k-slot l/16); rows >= M feed unused columns of D and read row M-1
        const uint16_t* bh = xs + (size_t)min(li, a.M - 1) * row_e + lq * 8 + s_begin * 32;
        const uint16_t* bl = bh + (size_t)a.M * row_e;
        int j = 0;
        // whole groups whose prefetches (steps j + DEPTH + u) are all inside the range: no clamps, no selects
        for (; j + 2 * DEPTH <= n; j += DEPTH) {
            woff += DEPTH * 4096;
            uint4 Bh[DEPTH], Bl[DEPTH];                           // the group's B operands, all LDS reads in flight together
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                Bh[u] = *reinterpret_cast<const uint4*>(bh + (j + u) * 32);
                Bl[u] = *reinterpret_cast<const uint4*>(bl + (j + u) * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const bf16x8 A = __builtin_bit_cast(bf16x8, rw[u]);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, Bh[u]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, Bl[u]), acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);                // keep the refill behind its MFMAs: same registers, no copies
                rw[u] = ldg16((const uint16_t*)(wb + woff + u * 4096));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // last groups: prefetches clamped to the last step, steps past the end meet zero weights
        for (; j < n; j += DEPTH) {
            woff += DEPTH * 4096;
            uint4 Bh[DEPTH], Bl[DEPTH];
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int sj = min(j + u, n - 1);
                Bh[u] = *reinterpret_cast<const uint4*>(bh + sj * 32);
                Bl[u] = *reinterpret_cast<const uint4*>(bl + sj * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                uint4 wv = rw[u];
                if (j + u >= n) wv = make_uint4(0u, 0u, 0u, 0u);
                const bf16x8 A = __builtin_bit_cast(bf16x8, wv);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, Bh[u]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, Bl[u]), acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                const int st = u - max(j + DEPTH + u - (n - 1), 0);      // relative to woff; negative = back inside the range
                rw[u] = ldg16((const uint16_t*)(wb + woff + st * 4096));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    *reinterpret_cast<f32x4*>(&red[wave][lane * 4]) = acc;
    __syncthreads();
    if (wave != 0) return;
    // lane holds D[column n0 + 4*lq + e][row li]
    f32x4 t = {0.f, 0.f, 0.f, 0.f}, t2 = {0.f, 0.f, 0.f, 0.f};
    for (int v = 0; v < WS; ++v) {
        const f32x4 p = *reinterpret_cast<const f32x4*>(&red[v][lane * 4]);
        t[0] += p[0]; t[1] += p[1]; t[2] += p[2]; t[3] += p[3];
    }
    if (EPI == EPI_SWIGLU)
        for (int v = WS; v < 2 * WS; ++v) {
            const f32x4 p = *reinterpret_cast<const f32x4*>(&red[v][lane * 4]);
            t2[0] += p[0]; t2[1] += p[1]; t2[2] += p[2]; t2[3] += p[3];
        }
    float rscale = 1.f;
    if (EPI != EPI_RESID) {      // r = rsqrt(mean square + eps) of the lane's input row
        float mine = 0.f;
#pragma unroll
        for (int mm = 0; mm < DEC_MAX_ROWS; ++mm) {
            const float tot = wsum(ssr[mm]);
            if (li == mm) mine = tot;
        }
        rscale = 1.0f / sqrtf(mine / (float)a.K + a.eps);
    }
    if (EPI == EPI_RESID) {
        float ss = 0.f;
        if (row_ok) {
            float* xp = a.x + (size_t)li * a.N + c;
            float4 xv = x_old;
            xv.x += t[0]; xv.y += t[1]; xv.z += t[2]; xv.w += t[3];
            *reinterpret_cast<float4*>(xp) = xv;
            ss = xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
            if (a.gain_next) {
                const float4 g = g_next;
                store_planes4(a.out_planes, a.out_plane, (size_t)li * a.N + c, xv.x * g.x, xv.y * g.y, xv.z * g.z, xv.w * g.w);
            }
        }
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (row_ok && lq == 0 && a.ssq_out) a.ssq_out[(size_t)li * (a.N / 16) + blockIdx.x] = ss;
    } else if (EPI == EPI_SWIGLU) {
        if (row_ok) {
            float h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float g = t[e] * rscale, u = t2[e] * rscale;
                h[e] = g / (1.0f + __expf(-g)) * u;
            }
            store_planes4(a.out_planes, a.out_plane, (size_t)li * a.N + c, h[0], h[1], h[2], h[3]);
        }
    } else {
        if (row_ok) {
            const int nq = a.H * a.hd, nkv = a.KVH * a.hd;
            const int p = p_row, b = li / a.q_len;
            float v[4] = {t[0] * rscale, t[1] * rscale, t[2] * rscale, t[3] * rscale};
            if (c < nq + nkv) {
                const int hc = c & hd_mask;
                const float2 c0 = rc0, c1 = rc1;
                const float r0 = v[0] * c0.x - v[1] * c0.y, r1 = v[0] * c0.y + v[1] * c0.x;
                const float r2 = v[2] * c1.x - v[3] * c1.y, r3 = v[2] * c1.y + v[3] * c1.x;
                if (c < nq) {
                    *reinterpret_cast<float4*>(a.q_out + (size_t)li * nq + c) = make_float4(r0, r1, r2, r3);
                } else if (p >= 0) {
                    const int kh = (c - nq) >> (__ffs(a.hd) - 1);
                    uint16_t* dst = a.k_cache + (((size_t)b * a.KVH + kh) * a.cache_len + p) * a.hd + hc;
                    *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)from_f<uint16_t>(r0) | ((uint32_t)from_f<uint16_t>(r1) << 16),
                                                                (uint32_t)from_f<uint16_t>(r2) | ((uint32_t)from_f<uint16_t>(r3) << 16));
                }
            } else if (p >= 0) {
                const int cv = c - nq - nkv;
                const int vh = cv >> (__ffs(a.hd) - 1), hc = cv & hd_mask;
                uint16_t* base = a.v_cache + ((size_t)b * a.KVH + vh) * (size_t)a.cache_len * a.hd;
#pragma unroll
                for (int e = 0; e < 4; ++e) base[v_index<uint16_t>(p, hc + e, a.hd)] = from_f<uint16_t>(v[e]);
            }
        }
    }
}

// ---- fused projections for a few more rows of a wide model (verification of one sequence) -----------------
// Between 3 and 16 rows the activations are too many to stage whole in every 16-column workgroup, and the 16-row
// kernel above needs a consumer kernel per projection for its split-K partial sums.  On a wide model (about as many
// 16-column units per projection as compute units, or more) there is a third way: one workgroup per compute unit
// owns up to ROWS_UMAX consecutive units over the WHOLE K range, its 8 wavefronts split K, every wavefront streams
// its k steps of all the units and loads the matching activations straight into the MFMA B operand (rows < M only;
// each k slice is read by one wavefront, so LDS would buy nothing, and the B registers are shared by the units),
// the accumulators meet in LDS and wavefront v finishes unit v with the consumer's work: RMS scale + RoPE + q out +
// K/V cache write (EPI_QKV), silu(r g) * (r u) as planes (EPI_SWIGLU, a unit being the gate and the up tile of the
// same 16 columns), residual add + planes of gain_next .* x + the unit's sums of squares (EPI_RESID).  No partial
// sums, no consumer kernel.  The activation planes are tiled (xt_index): with the rows of a k step in 16 different
// cache lines a projection with ONE unit per workgroup (O, down), whose activations are as many bytes as its
// weights, ran a third slower (down projection, 9 rows: 27 against 21 us).
constexpr int ROWS_UMAX = 4;
constexpr int rows_depth(int nt) { return nt <= 4 ? 4 : 2; }   // k steps in flight per wavefront (3 measured a third slower than 2 or 4)

template <int EPI, int NU>
__device__ __forceinline__ void rows_body(const DecArgs& a, const int u0, float* __restrict__ red) {
    constexpr int PER = EPI == EPI_SWIGLU ? 2 : 1, NT = NU * PER, DEPTH = rows_depth(NT);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const bool row_ok = li < a.M;
    const int m = min(li, a.M - 1);
    // what the epilogue needs from memory is requested ahead of the operand streams (wavefront v finishes unit v)
    const int c = (u0 + min(wave, NU - 1)) * 16 + 4 * lq;         // the lane's four output columns there
    const int hd_mask = a.hd - 1;
    float2 rc0 = make_float2(1.f, 0.f), rc1 = make_float2(1.f, 0.f);
    float4 x_old = make_float4(0.f, 0.f, 0.f, 0.f), g_next = make_float4(0.f, 0.f, 0.f, 0.f);
    int p_row = -1;
    if (wave < NU) {
        if (EPI == EPI_QKV) {
            p_row = a.pos[m];
            const int hc = c & hd_mask;
            rc0 = a.rope[(size_t)m * (a.hd / 2) + hc / 2];
            rc1 = a.rope[(size_t)m * (a.hd / 2) + hc / 2 + 1];
        }
        if (EPI == EPI_RESID) {
            x_old = *reinterpret_cast<const float4*>(a.x + (size_t)m * a.N + c);
            if (a.gain_next) g_next = *reinterpret_cast<const float4*>(a.gain_next + c);
        }
    }
    // The input rows' sums of squares come in ssq_tiles pieces per row (4 from the residual kernel, K/16 from an
    // EPI_RESID projection): the lanes (row li, lq) of all wavefronts share the pieces, 8 independent loads each
    // (256 pieces), added up behind the operand streams and combined through LDS with the accumulators.
    float sv[8];
    if (EPI != EPI_RESID) {
#pragma unroll
        for (int i = 0; i < 8; ++i) sv[i] = a.ssq_in[(size_t)m * a.ssq_tiles + min(wave * 4 + lq + 32 * i, a.ssq_tiles - 1)];
    }
    const int steps = a.K / 32;
    const int s_begin = (wave * steps) >> 3, s_end = ((wave + 1) * steps) >> 3;
    const int n = s_end - s_begin, nn = max(n, 1) - 1;
    const int sb = n > 0 ? s_begin : 0;                            // a wavefront without k steps re-reads step 0 and ignores it
    const char* wp[NT];                                            // the wavefront's first k step of every tile (uniform)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int local = (u0 + t / PER) * 16;
        const void* mat;
        if (EPI == EPI_SWIGLU) mat = a.w[t % PER];
        else {
            int seg = 0;
            if (a.w[1] && local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (a.w[2] && local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
            mat = a.w[seg];
        }
        wp[t] = reinterpret_cast<const char*>(mat) + ((size_t)(local >> 6) * 64 * a.K + ((local >> 4) & 3) * 512 + (size_t)sb * 2048) * 2;
    }
    const uint32_t loff = lane * 16;                               // a k step of a tile is one contiguous kilobyte, 16 bytes per lane
    const uint16_t* bh = a.xh + (size_t)sb * 512 + m * 32 + lq * 8;         // tiled planes (xt_index): a k step is 512 elements
    const uint16_t* bl = bh + a.x_plane;
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint4 rw[DEPTH][NT], Bh[DEPTH], Bl[DEPTH];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
        const int sj = min(u, nn);
        Bh[u] = make_uint4(0u, 0u, 0u, 0u); Bl[u] = make_uint4(0u, 0u, 0u, 0u);
        if (row_ok) { Bh[u] = ldg16(bh + sj * 512); Bl[u] = ldg16(bl + sj * 512); }    // rows >= M stay zero
#pragma unroll
        for (int t = 0; t < NT; ++t) rw[u][t] = ldg16(reinterpret_cast<const uint16_t*>(wp[t] + loff + sj * 4096));
    }
    for (int j = 0; j < n; j += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const bool live = j + u < n;                           // steps past the end meet zero weights
            const bf16x8 vh = __builtin_bit_cast(bf16x8, Bh[u]), vl = __builtin_bit_cast(bf16x8, Bl[u]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                uint4 wv = rw[u][t];
                if (!live) wv = make_uint4(0u, 0u, 0u, 0u);
                const bf16x8 A = __builtin_bit_cast(bf16x8, wv);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, vh, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, vl, acc[t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);                     // keep the refill behind its MFMAs: same registers, no copies
            const int sj = min(j + DEPTH + u, nn);                 // prefetches clamped to the last step
            if (row_ok) { Bh[u] = ldg16(bh + sj * 512); Bl[u] = ldg16(bl + sj * 512); }
#pragma unroll
            for (int t = 0; t < NT; ++t) rw[u][t] = ldg16(reinterpret_cast<const uint16_t*>(wp[t] + loff + sj * 4096));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) *reinterpret_cast<f32x4*>(&red[(wave * NT + t) * 256 + lane * 4]) = acc[t];
    float* ssred = red + 8 * NT * 256;                             // [8 wavefronts][16 rows]
    if (EPI != EPI_RESID) {
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) part += wave * 4 + lq + 32 * i < a.ssq_tiles ? sv[i] : 0.f;
        for (int t = wave * 4 + lq + 256; t < a.ssq_tiles; t += 32) part += a.ssq_in[(size_t)m * a.ssq_tiles + t];
        part += __shfl_xor(part, 16, 64);
        part += __shfl_xor(part, 32, 64);
        if (lq == 0) ssred[wave * 16 + li] = part;
    }
    __syncthreads();
    if (wave >= NU) return;
    // lane holds D[column c + e][row li] of unit `wave`
    f32x4 t1 = {0.f, 0.f, 0.f, 0.f}, t2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const f32x4 p = *reinterpret_cast<const f32x4*>(&red[(v * NT + wave * PER) * 256 + lane * 4]);
        t1[0] += p[0]; t1[1] += p[1]; t1[2] += p[2]; t1[3] += p[3];
        if (EPI == EPI_SWIGLU) {
            const f32x4 q = *reinterpret_cast<const f32x4*>(&red[(v * NT + wave * PER + 1) * 256 + lane * 4]);
            t2[0] += q[0]; t2[1] += q[1]; t2[2] += q[2]; t2[3] += q[3];
        }
    }
    if (EPI == EPI_RESID) {
        float ss = 0.f;
        if (row_ok) {
            float4 xv = x_old;
            xv.x += t1[0]; xv.y += t1[1]; xv.z += t1[2]; xv.w += t1[3];
            *reinterpret_cast<float4*>(a.x + (size_t)li * a.N + c) = xv;
            ss = xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
            if (a.gain_next)
                store_planes4(a.out_planes, a.out_plane, a.out_tiled ? xt_index(li, c) : (size_t)li * a.N + c,
                              xv.x * g_next.x, xv.y * g_next.y, xv.z * g_next.z, xv.w * g_next.w);
        }
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (row_ok && lq == 0 && a.ssq_out) a.ssq_out[(size_t)li * (a.N / 16) + (c >> 4)] = ss;
        return;
    }
    if (!row_ok) return;
    float ssq = 0.f;
#pragma unroll
    for (int v = 0; v < 8; ++v) ssq += ssred[v * 16 + li];
    const float rscale = 1.0f / sqrtf(ssq / (float)a.K + a.eps);  // r = rsqrt(mean square + eps) of the lane's input row
    if (EPI == EPI_SWIGLU) {
        float h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float g = t1[e] * rscale, u = t2[e] * rscale;
            h[e] = g / (1.0f + __expf(-g)) * u;
        }
        store_planes4(a.out_planes, a.out_plane, a.out_tiled ? xt_index(li, c) : (size_t)li * a.N + c, h[0], h[1], h[2], h[3]);
    } else {
        const int nq = a.H * a.hd, nkv = a.KVH * a.hd;
        const int p = p_row, b = li / a.q_len;
        const float v[4] = {t1[0] * rscale, t1[1] * rscale, t1[2] * rscale, t1[3] * rscale};
        if (c < nq + nkv) {
            const int hc = c & hd_mask;
            const float r0 = v[0] * rc0.x - v[1] * rc0.y, r1 = v[0] * rc0.y + v[1] * rc0.x;
            const float r2 = v[2] * rc1.x - v[3] * rc1.y, r3 = v[2] * rc1.y + v[3] * rc1.x;
            if (c < nq) {
                *reinterpret_cast<float4*>(a.q_out + (size_t)li * nq + c) = make_float4(r0, r1, r2, r3);
            } else if (p >= 0) {
                const int kh = (c - nq) >> (__ffs(a.hd) - 1);
                uint16_t* dst = a.k_cache + (((size_t)b * a.KVH + kh) * a.cache_len + p) * a.hd + hc;
                *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)from_f<uint16_t>(r0) | ((uint32_t)from_f<uint16_t>(r1) << 16),
                                                            (uint32_t)from_f<uint16_t>(r2) | ((uint32_t)from_f<uint16_t>(r3) << 16));
            }
        } else if (p >= 0) {
            const int cv = c - nq - nkv;
            const int vh = cv >> (__ffs(a.hd) - 1), hc = cv & hd_mask;
            uint16_t* base = a.v_cache + ((size_t)b * a.KVH + vh) * (size_t)a.cache_len * a.hd;
#pragma unroll
            for (int e = 0; e < 4; ++e) base[v_index<uint16_t>(p, hc + e, a.hd)] = from_f<uint16_t>(v[e]);
        }
    }
}

// `units` units are dealt to the workgroups in consecutive runs of TU or TU - 1 (host: ceil(units / grid) == TU, grid <= units)
template <int EPI, int TU>
__global__ __launch_bounds__(512) void gemm_rows_kernel(DecArgs a, int units) {
    extern __shared__ __attribute__((aligned(16))) float rows_red[];      // [8 wavefronts][tiles][256]
    const int G = gridDim.x, b = blockIdx.x;
    const int base = units / G, rem = units - base * G;
    const int nu = base + (b < rem ? 1 : 0), u0 = b * base + min(b, rem);
    if (nu == TU) rows_body<EPI, TU>(a, u0, rows_red);
    else if (TU > 1 && nu == TU - 1) rows_body<EPI, (TU > 1 ? TU - 1 : 1)>(a, u0, rows_red);
}

// Split-K factor of the 16-row kernel: the smallest power of two that gives about 450 workgroups (two per
// compute unit keep enough loads in flight; measured on the 7B shapes, more splits only add partial sums
// for the consumer kernels to read), with at least 256 columns per split.
static int m16_splits(int N, int K) {
    const int tiles = (N + 63) / 64;
    int ks = 1;
    while (ks * tiles < 448) ks *= 2;
    const int cap = K / 256 > 1 ? K / 256 : 1;
    if (ks > cap) ks = cap;
    const int kper = ((K + ks - 1) / ks + 31) / 32 * 32;
    return (K + kper - 1) / kper;
}

// ---- GEMM, fp32 (plumbing configuration): one wavefront per output column, lanes stride K ----------
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    if (n >= a.N) return;
    int seg = 0, local = n;
    if (local >= a.seg_rows[0]) { local -= a.seg_rows[0]; seg = 1; if (local >= a.seg_rows[1]) { local -= a.seg_rows[1]; seg = 2; } }
    const float* w0 = reinterpret_cast<const float*>(a.w[seg]) + (size_t)local * a.K;
    const float* x = reinterpret_cast<const float*>(a.x);
    for (int m0 = 0; m0 < a.M; m0 += 8) {
        float acc[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = 0.f;
        for (int k = lane; k < a.K; k += 64) {
            const float wv = w0[k];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float xv = (m0 + r < a.M) ? x[(size_t)(m0 + r) * a.K + k] : 0.f;
                acc[r] = fmaf(xv, wv, acc[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float v = wsum(acc[r]);
            if (lane == 0 && m0 + r < a.M) reinterpret_cast<float*>(a.out)[(size_t)(m0 + r) * a.ldo + n] = v;
        }
    }
}

// Weight tiles per wavefront of the many-row kernel: two from 97 rows on (halves the LDS reads per weight byte,
// which is what bounds the kernel there).
int gemm_splits(int dtype, int N, int K, int M) {
    if (dtype != BS_BF16) return 1;
    if (M <= 16) return m16_splits(N, K);
    const int stages = (K + 255) / 256;
    if (M > 32 && K % 32 == 0) {
        // 256 weight rows per workgroup, one workgroup per compute unit: as many splits as fill the chip once and no
        // more -- every further split writes and re-reads megabytes of partial sums
        const int tiles = (N + 255) / 256 * ((M + 255) / 256);       // blocks of 256 rows share a launch
        int ks = 256 / tiles;
        if (ks < 1) {
            // more tiles than compute units: splitting can still even out the last, partly filled round of workgroups
            // (344 tiles: two rounds unsplit, three half-length rounds in two splits; measured 306 -> 262 us)
            ks = 1;
            double best = 1e30;
            for (int c = 1; c <= 4; ++c) {
                const double cost = (double)((tiles * c + 255) / 256) / c + 0.04 * (c - 1);
                if (cost < best) { best = cost; ks = c; }
            }
        }
        if (ks > stages) ks = stages;
        if (ks > 16) ks = 16;
        return ks < 1 ? 1 : ks;
    }
    const int tiles = (N + 63) / 64;
    int ks = (768 + tiles - 1) / tiles;
    if (ks > stages / 2) ks = stages / 2;
    if (ks > 16) ks = 16;
    if (ks < 1) ks = 1;
    return ks;
}

// A kernel launch that, while the measurement hook is on (e0 != nullptr), carries its own start and stop events: they
// take the dispatch's begin and end times, so the elapsed time is the kernel's and nothing else (two events recorded
// around a launch also measure 2-3 us of dispatch).
#define BS_LAUNCH_TIMED(kernel, grid, block, lds, stream, e0, e1, ...) \
    do { if (e0) hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)(lds), stream, e0, e1, 0, __VA_ARGS__); \
         else hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__); } while (0)

// ---- optional per-launch timing of the weight-streaming GEMM (measurement hook) ----------------------
struct GemmProfile {
    bool on = false;
    std::vector<hipEvent_t> ev;       // pairs (start, stop)
    std::vector<double> bytes;        // algorithmic bytes of each timed launch: the weight tile once
    std::vector<int> mt;
};
static GemmProfile g_prof;
static std::mutex g_prof_mutex;      // launches may come from several host threads

// Switching on starts an empty record; switching off drops the record and its events (collect first).
int profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof.on = on != 0;
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear(); g_prof.bytes.clear(); g_prof.mt.clear();
    return BS_OK;
}

// Events for one timed launch, or none when the record is off.  Events cannot be recorded into a stream capture: a
// launch that is being captured while the record is on is refused.
static int prof_events(hipStream_t s, hipEvent_t* e0, hipEvent_t* e1) {
    *e0 = nullptr; *e1 = nullptr;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof.on) return BS_OK;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    BS_HIP(hipStreamIsCapturing(s, &st));
    BS_REQUIRE(st == hipStreamCaptureStatusNone, BS_ESTATE, "per-launch timing is switched on while the stream is being captured: "
               "switch it off (bs_profile_enable(0)) before capturing");
    BS_HIP(hipEventCreate(e0));
    if (hipEventCreate(e1) != hipSuccess) { (void)hipEventDestroy(*e0); *e0 = nullptr; BS_FAIL(BS_EHIP, "hipEventCreate failed"); }
    return BS_OK;
}
static void prof_record(hipEvent_t e0, hipEvent_t e1, double bytes, int cls) {
    if (!e0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof.on) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return; }   // switched off in between
    g_prof.ev.push_back(e0); g_prof.ev.push_back(e1);
    g_prof.bytes.push_back(bytes);
    g_prof.mt.push_back(cls);
}

int profile_collect(int mt_filter, double* total_ms, double* total_bytes, long long* launches) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    double ms = 0.0, by = 0.0;
    long long n = 0;
    for (size_t i = 0; i < g_prof.bytes.size(); ++i) {
        if (mt_filter > 0 && g_prof.mt[i] != mt_filter) continue;
        BS_HIP(hipEventSynchronize(g_prof.ev[2 * i + 1]));
        float t = 0.f;
        BS_HIP(hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]));
        ms += t; by += g_prof.bytes[i]; ++n;
    }
    if (total_ms) *total_ms = ms;
    if (total_bytes) *total_bytes = by;
    if (launches) *launches = n;
    return BS_OK;
}

size_t packed_elems(int N, int K) { return (size_t)((N + 63) / 64) * 64 * (size_t)K; }

int launch_pack_weights(const void* src, void* dst, int N, int K, hipStream_t s) {
    BS_REQUIRE(K % 32 == 0 && N >= 1, BS_ESHAPE, "pack_weights: K=%d must be a multiple of 32", K);
    const size_t chunks = packed_elems(N, K) / 8;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)src, (uint16_t*)dst, N, K);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_gemm(int dtype, GemmArgs a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return BS_OK;
    BS_REQUIRE(!a.tiled || (dtype == BS_BF16 && a.K % 32 == 0 && (!a.w[1] || a.seg_rows[0] % 16 == 0) && (!a.w[2] || a.seg_rows[1] % 16 == 0)),
               BS_ESHAPE, "gemm: tiled weights need bf16, K %% 32 == 0 and stacked matrices whose row counts are multiples of 16");
    if (dtype == BS_F32) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((a.N + 3) / 4), dim3(256), 0, s, a);
        BS_LAUNCH_CHECK();
        return BS_OK;
    }
    const bool big_ok = a.K % 32 == 0;                              // the many-row kernel works in whole 32-column stages
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto prof_begin = [&]() -> int { return prof_events(s, &e0, &e1); };
    auto prof_end = [&](int mt) -> int {                            // classes by 16-row tiles: 1, 2, 4, 6, 8, 16
        prof_record(e0, e1, (double)a.N * (double)a.K * 2.0, mt <= 1 ? 1 : mt <= 2 ? 2 : mt <= 4 ? 4 : mt <= 6 ? 6 : mt <= 8 ? 8 : 16);
        return BS_OK;
    };
    int rc;
    if (big_ok && a.M > 32) {
        // 33 rows and more: one launch; beyond 256 rows several blocks of 256 rows share it (more workgroups per
        // weight tile instead of more splits of K)
        const int mt = a.M > GEMM_MAX_ROWS ? 16 : (a.M + 15) / 16;
        const int n_mb = (a.M + 255) / 256, groups = ((a.N + 255) / 256 + 7) / 8;      // whole groups of 8 weight tiles
        const dim3 grid(groups * 8 * n_mb, a.KS), block(64 * BIG_WAVES);
        if ((rc = prof_begin()) != BS_OK) return rc;
#define BS_BIG(MT) do { if (a.tiled) BS_LAUNCH_TIMED((gemm_bf16_big_kernel<MT, true>), grid, block, 0, s, e0, e1, a); \
                        else BS_LAUNCH_TIMED((gemm_bf16_big_kernel<MT, false>), grid, block, 0, s, e0, e1, a); } while (0)
        if (mt <= 4) BS_BIG(4);
        else if (mt <= 6) BS_BIG(6);
        else if (mt <= 8) BS_BIG(8);
        else if (mt <= 10) BS_BIG(10);
        else if (mt <= 12) BS_BIG(12);
        else if (mt <= 14) BS_BIG(14);
        else BS_BIG(16);
#undef BS_BIG
        BS_LAUNCH_CHECK();
        return prof_end(mt);
    }
    // up to 32 rows (or K not a multiple of 32: 32 rows at a time)
    const int max_rows = a.M <= 16 ? 16 : 32;
    for (int m0 = 0; m0 < a.M; m0 += max_rows) {
        GemmArgs c = a;
        c.M = (a.M - m0 < max_rows) ? a.M - m0 : max_rows;
        c.x = reinterpret_cast<const uint16_t*>(a.x) + (size_t)m0 * a.K;
        c.out = reinterpret_cast<float*>(a.out) + (size_t)m0 * a.ldo;
        const dim3 grid((a.N + 63) / 64, a.KS), block(256);
        const int kper = ((a.K + a.KS - 1) / a.KS + 31) / 32 * 32;      // columns per split, whole k slices
        if ((rc = prof_begin()) != BS_OK) return rc;
        // one 16-row weight tile per wavefront measured faster than two (3.7 vs 3.2 TB/s over the 7B layer shapes)
        if (a.M <= 16) {
            if (a.tiled) BS_LAUNCH_TIMED((gemm_bf16_m16_kernel<1, true>), grid, block, 0, s, e0, e1, c, kper);
            else BS_LAUNCH_TIMED((gemm_bf16_m16_kernel<1, false>), grid, block, 0, s, e0, e1, c, kper);
        } else {
            if (a.tiled) BS_LAUNCH_TIMED((gemm_bf16_kernel<2, 1, 256, true>), grid, block, 0, s, e0, e1, c);
            else BS_LAUNCH_TIMED((gemm_bf16_kernel<2, 1, 256, false>), grid, block, 0, s, e0, e1, c);
        }
        BS_LAUNCH_CHECK();
        if ((rc = prof_end((c.M + 15) / 16)) != BS_OK) return rc;
    }
    return BS_OK;
}

// ---- RoPE + KV append -----------------------------------------------------------------------------
// grid (M, H + 2*KVH); thread = one rotation pair.  Row layout of the projection: [q heads | k heads | v heads],
// given as split-K partials that are summed here.  q stays fp32; k and v are rounded to the cache dtype.
template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ part, int ks, size_t ks_stride, const int32_t* __restrict__ pos,
                               const float2* __restrict__ rope, int q_len, int H, int KVH, int hd, int max_len,
                               float* __restrict__ q_out, T* __restrict__ k_cache, T* __restrict__ v_cache,
                               const float* __restrict__ ssq, int nchunks, float inv_d, float eps) {
    const int m = blockIdx.x, head = blockIdx.y, i = threadIdx.x;       // i < hd/2
    const int p = pos[m];
    const int b = m / q_len;
    const int ld = (H + 2 * KVH) * hd;
    const float* src = part + (size_t)m * ld + (size_t)head * hd;
    float x0 = 0.f, x1 = 0.f;
    for (int s = 0; s < ks; ++s) {
        const float2 v = *reinterpret_cast<const float2*>(src + (size_t)s * ks_stride + 2 * i);
        x0 += v.x; x1 += v.y;
    }
    {
        const float rs = row_rscale(ssq, nchunks, m, inv_d, eps);      // the input rows' RMS scale, if it was deferred
        x0 *= rs; x1 *= rs;
    }
    if (head < H + KVH) {
        const float2 cs = rope[(size_t)m * (hd / 2) + i];
        const float r0 = x0 * cs.x - x1 * cs.y, r1 = x0 * cs.y + x1 * cs.x;
        if (head < H) {
            float* dst = q_out + (size_t)m * H * hd + (size_t)head * hd;
            dst[2 * i] = r0; dst[2 * i + 1] = r1;
        } else if (p >= 0) {
            T* dst = k_cache + (((size_t)b * KVH + (head - H)) * max_len + p) * hd;
            dst[2 * i] = from_f<T>(r0); dst[2 * i + 1] = from_f<T>(r1);
        }
    } else if (p >= 0) {
        T* base = v_cache + ((size_t)b * KVH + (head - H - KVH)) * (size_t)max_len * hd;
        base[v_index<T>(p, 2 * i, hd)] = from_f<T>(x0);
        base[v_index<T>(p, 2 * i + 1, hd)] = from_f<T>(x1);
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
__global__ __launch_bounds__(256) void attn_kernel(const float* __restrict__ q, const T* __restrict__ k_cache,
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
    const size_t pstride = (size_t)hd + 4;       // o[hd], max, sum, 2 pad: rows stay 16-byte aligned
    if (pos0 < 0) {                                // sequence skipped: empty partials
        for (int idx = threadIdx.x; idx < q_len; idx += 256) {
            float* dst = part + ((((size_t)(m_first + idx)) * H + h) * n_splits + split) * pstride;
            dst[hd] = -INFINITY; dst[hd + 1] = 0.f;
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
            qs[r][d] = (r < nr) ? q[((size_t)(m_first + r0 + r) * H + h) * hd + d] * scale : 0.f;
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
                    const int vk = t * 64 + kk + u;
                    v0[u] = (okk && d0 < hd) ? to_f(vb[v_index<T>(vk, d0, hd)]) : 0.f;
                    v1[u] = (okk && d1 < hd) ? to_f(vb[v_index<T>(vk, d1, hd)]) : 0.f;
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
            dst[d] = o;
            if (d == 0) { dst[hd] = mm; dst[hd + 1] = l; }
        }
    }
}

// ---- attention, bf16 cache, MFMA ---------------------------------------------------------------------
// grid (n_splits, KVH, B), 4 wavefronts.  Rows of the score matrix = the q_len query positions of the
// H/KVH query heads that share this kv head (16 rows per MFMA tile).  The wavefronts take the 32-key
// blocks of their split in turn:
//   S^T = K . Q^T      A = K rows straight from the cache, B = Q (fp32 queries as a bf16 hi/lo pair)
//   online softmax     a row lives in one lane column (l % 16); its 32 scores sit in 4 lanes -> 2 shuffles
//   O^T += V^T . P^T   A = transposed V block (one 16-byte load per lane), B = P^T taken from the score
//                      accumulators as they are (hi/lo pair), no LDS, no transposes
// Bytes: every K and V element is read once per 16 rows (per 32 with two tiles per wavefront, below).  Un-normalised
// partials (m, l, o[hd]) per split.
// NT = 16-row tiles a wavefront holds at the same time: every K and V block it loads is multiplied with all of them.
// With grouped queries a verification pass has G * (gamma + 1) rows per kv head, more than one tile from 17 rows on, and a
// second workgroup for the second tile walks the whole cache a second time (batch 32, 8192 cached keys, 24 rows: 3.7
// TB/s of distinct K/V bytes against 5.3 with one tile).  Two tiles take about 320 registers, one wavefront per SIMD;
// its next block is therefore requested before the current one is multiplied (two register sets, loop unrolled by two;
// two blocks ahead measured the same).
// Combining the key splits inside this kernel (mg.cells != null; one row tile, all workgroups resident together: host
// check): a workgroup hands its partial over in exchange cells instead of `part`, then the workgroup of split s combines,
// for the rows r = S-1-s, 2S-1-s, ... of its head group (S splits; the last splits hold the fewest keys, often none), the
// partials of all splits as they arrive (bounded polls) and writes the attention output planes -- the hand-over costs
// about two microseconds where a merge kernel costs five.
// The cells are all zero when the pass starts (prep kernel) and every layer hands over under its own flag.
struct AttnMerge {
    void* cells;                 // [M][H][n_splits][HD + 4] cells: o[HD], max, sum, 2 pad
    uint16_t* out; size_t plane; // attention output planes; tiled: in the layout of the whole-K projections (xt_index)
    int tiled;
    unsigned flag, spin_limit;
    int32_t* status;             // bit 16: a poll ran out of patience
};

template <int HD, int NT>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const float* __restrict__ q, const uint16_t* __restrict__ k_cache,
                                                        const uint16_t* __restrict__ v_cache,
                                                        const int32_t* __restrict__ pos, int q_len, int H, int KVH,
                                                        int cache_len, float scale, float* __restrict__ part, int n_splits,
                                                        uint16_t* __restrict__ direct_out, size_t plane, AttnMerge mg) {
    constexpr int DS = HD / 32, DT = HD / 16;
    constexpr int PC = HD + 4;                   // cells of one partial
    __shared__ float wm[4][16], wl[4][16];
    __shared__ float wo[4][16][HD + 1];
    // blockIdx.x = (group of NT row tiles, split of the keys): with many query rows (a prompt chunk) the groups are
    // spread over workgroups and the keys over few splits; with one group all of gridDim.x are key splits
    const int split = blockIdx.x % n_splits, rt = blockIdx.x / n_splits, n_rt = gridDim.x / n_splits;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int G = H / KVH, R = G * q_len;
    const int m_first = b * q_len;
    const int pos0 = pos[m_first];
    const size_t pstride = (size_t)HD + 4;       // o[HD], max, sum, 2 pad: rows stay 16-byte aligned
    if (pos0 < 0) {                                  // sequence skipped: empty partials (zeros when writing the output itself)
        if (direct_out) {
            for (int idx = threadIdx.x + rt * 256; idx < R * HD; idx += 256 * n_rt) {
                const int r = idx / HD, d = idx % HD;
                Act<uint16_t>::store(direct_out, plane, ((size_t)(m_first + r % q_len) * H + kvh * G + r / q_len) * HD + d, 0.f);
            }
            return;
        }
        if (NT == 1 && mg.cells) {                   // no workgroup of this sequence polls: the rows' owners write zeros
            for (int rr = n_splits - 1 - split; rr < R; rr += n_splits) {
                const int m = m_first + rr % q_len, head = kvh * G + rr / q_len;
                for (int d = threadIdx.x; d < HD; d += 256)
                    Act<uint16_t>::store(mg.out, mg.plane, mg.tiled ? xt_index(m, head * HD + d) : ((size_t)m * H + head) * HD + d, 0.f);
            }
            return;
        }
        for (int r = threadIdx.x; r < R; r += 256) {
            const int g = r / q_len, qi = r % q_len;
            float* dst = part + ((((size_t)(m_first + qi)) * H + kvh * G + g) * n_splits + split) * pstride;
            dst[HD] = -INFINITY; dst[HD + 1] = 0.f;
        }
        return;
    }
    const int n_keys = pos0 + q_len;
    const uint16_t* kb = k_cache + ((size_t)b * KVH + kvh) * (size_t)cache_len * HD;
    const uint16_t* vb = v_cache + ((size_t)b * KVH + kvh) * (size_t)cache_len * HD;

    for (int r0 = rt * 16 * NT; r0 < R; r0 += 16 * NT * n_rt) {
        // keys any row of this group may see (causal): up to the group's latest query position
        const int r_last = min(r0 + 16 * NT - 1, R - 1);
        const int qi_max = (r0 / q_len == r_last / q_len) ? r_last % q_len : q_len - 1;
        const int nblk = (pos0 + qi_max + 1 + 31) / 32;
        const int per = (nblk + n_splits - 1) / n_splits;
        const int b_begin = split * per, b_end = min(nblk, b_begin + per);
        bool rvalid[NT];
        int row_pos[NT];
        uint4 qh[NT][DS], ql[NT][DS];
        float m_run[NT], l_run[NT];
        f32x4 o[NT][DT];
#pragma unroll
        for (int x = 0; x < NT; ++x) {
            const int row = r0 + 16 * x + li;
            rvalid[x] = row < R;
            const int g = rvalid[x] ? row / q_len : 0, qi = rvalid[x] ? row % q_len : 0;
            row_pos[x] = pos0 + qi;
            const float* qrow = q + ((size_t)(m_first + qi) * H + kvh * G + g) * HD;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                float v[8];
                const float4 a = *reinterpret_cast<const float4*>(qrow + ds * 32 + lq * 8);
                const float4 c = *reinterpret_cast<const float4*>(qrow + ds * 32 + lq * 8 + 4);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c.x; v[5] = c.y; v[6] = c.z; v[7] = c.w;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = rvalid[x] ? v[e] * scale : 0.f;
                split8(v, qh[x][ds], ql[x][ds]);
            }
            m_run[x] = -INFINITY; l_run[x] = 0.f;
#pragma unroll
            for (int t = 0; t < DT; ++t) o[x][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        auto fetch = [&](int blk, uint4 (&kf)[2][DS], uint4 (&vf)[DT]) {
            const int key0 = blk * 32;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int krow = min(key0 + t * 16 + li, n_keys - 1);
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) kf[t][ds] = ldg16(kb + (size_t)krow * HD + ds * 32 + lq * 8);
            }
#pragma unroll
            for (int t = 0; t < DT; ++t) vf[t] = ldg16(vb + ((size_t)blk * HD + t * 16 + li) * 32 + lq * 8);
        };
        auto block = [&](int blk, uint4 (&kf)[2][DS], uint4 (&vf)[DT]) {
            const int key0 = blk * 32;
            // ---- values: keys past n_keys may hold anything, even NaN patterns: zero them ----
            if (key0 + 32 > n_keys) {
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    uint32_t w[4] = {vf[t].x, vf[t].y, vf[t].z, vf[t].w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int key = key0 + (e >> 2) * 16 + 4 * lq + (e & 3);
                        if (key >= n_keys) w[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                    }
                    vf[t] = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
#pragma unroll
            for (int x = 0; x < NT; ++x) {
                // ---- scores of 32 keys x 16 rows ----
                f32x4 sc[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) {
                        const bf16x8 A = __builtin_bit_cast(bf16x8, kf[t][ds]);
                        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, qh[x][ds]), sc[t], 0, 0, 0);
                        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, ql[x][ds]), sc[t], 0, 0, 0);
                    }
                }
                // lane holds S^T[key0 + 16t + 4lq + e][row li]
                float sv[8];
                float bm = -INFINITY;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int key = key0 + t * 16 + 4 * lq + e;
                        const bool vis = rvalid[x] && key < n_keys && key <= row_pos[x];       // causal
                        sv[t * 4 + e] = vis ? sc[t][e] : -INFINITY;
                        bm = fmaxf(bm, sv[t * 4 + e]);
                    }
                bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
                bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
                const float m_new = fmaxf(m_run[x], bm);
                float pv[8];
                float alpha = 1.f, psum = 0.f;
                if (m_new == -INFINITY) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) pv[e] = 0.f;
                } else {
                    alpha = __expf(m_run[x] - m_new);
#pragma unroll
                    for (int e = 0; e < 8; ++e) { pv[e] = __expf(sv[e] - m_new); psum += pv[e]; }
                }
                l_run[x] = l_run[x] * alpha + psum;
                m_run[x] = m_new;
                uint4 ph, pl;
                split8(pv, ph, pl);
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    o[x][t][0] *= alpha; o[x][t][1] *= alpha; o[x][t][2] *= alpha; o[x][t][3] *= alpha;
                    const bf16x8 A = __builtin_bit_cast(bf16x8, vf[t]);
                    o[x][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, ph), o[x][t], 0, 0, 0);
                    o[x][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, pl), o[x][t], 0, 0, 0);
                }
            }
        };
        if constexpr (NT == 1) {
            for (int blk = b_begin + wave; blk < b_end; blk += 4) {
                uint4 kf[2][DS], vf[DT];
                fetch(blk, kf, vf);
                block(blk, kf, vf);
            }
        } else if (b_begin + wave < b_end) {
            // a request past the wavefront's last block repeats that block: in bounds, never used
            const int blk_last = b_begin + wave + ((b_end - 1 - b_begin - wave) >> 2) * 4;
            uint4 kf0[2][DS], vf0[DT], kf1[2][DS], vf1[DT];
            fetch(b_begin + wave, kf0, vf0);
            for (int blk = b_begin + wave; blk < b_end; blk += 8) {
                fetch(min(blk + 4, blk_last), kf1, vf1);
                block(blk, kf0, vf0);
                if (blk + 4 >= b_end) break;
                fetch(min(blk + 8, blk_last), kf0, vf0);
                block(blk + 4, kf1, vf1);
            }
        }
        // ---- combine the 4 wavefronts, one tile at a time: lane holds O^T[d = 16t + 4lq + e][row li] ----
#pragma unroll
        for (int x = 0; x < NT; ++x) {
            const int rbase = r0 + 16 * x;
            if (rbase >= R) break;
            float lr = l_run[x];
            lr += __shfl_xor(lr, 16, 64);
            lr += __shfl_xor(lr, 32, 64);
            __syncthreads();
            if (lq == 0) { wm[wave][li] = m_run[x]; wl[wave][li] = lr; }
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) wo[wave][li][t * 16 + 4 * lq + e] = o[x][t][e];
            __syncthreads();
            for (int idx = threadIdx.x; idx < 16 * HD; idx += 256) {
                const int r = idx / HD, d = idx % HD;
                if (rbase + r >= R) continue;
                const float mm = fmaxf(fmaxf(wm[0][r], wm[1][r]), fmaxf(wm[2][r], wm[3][r]));
                float ov = 0.f, lv = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float f = (wm[w][r] == -INFINITY) ? 0.f : __expf(wm[w][r] - mm);
                    ov += wo[w][r][d] * f;
                    lv += wl[w][r] * f;
                }
                const int gg = (rbase + r) / q_len, qq = (rbase + r) % q_len;
                if (direct_out) {                    // a single split of the keys: this is the attention output
                    Act<uint16_t>::store(direct_out, plane, ((size_t)(m_first + qq) * H + kvh * G + gg) * HD + d, lv > 0.f ? ov / lv : 0.f);
                    continue;
                }
                if (NT == 1 && mg.cells) {           // hand the partial over in cells
                    const DevBuf bc = dev_buf(mg.cells);
                    const int c0 = (((m_first + qq) * H + kvh * G + gg) * n_splits + split) * PC;
                    st_cell1(bc, c0 + d, ov, mg.flag);
                    if (d == 0) st_cells2(bc, c0 + HD, mm, lv, mg.flag);
                    continue;
                }
                float* dst = part + ((((size_t)(m_first + qq)) * H + kvh * G + gg) * n_splits + split) * pstride;
                dst[d] = ov;
                if (d == 0) { dst[HD] = mm; dst[HD + 1] = lv; }
            }
        }
    }
    if constexpr (NT == 1) {
        if (!mg.cells) return;
        // ---- combine the splits of this workgroup's rows: lane = (head-dim element d, share sp0 of the splits) ----
        constexpr int P = 256 / HD;                  // HD threads per share; sp0 is uniform in a wavefront
        constexpr int MU = 8;                        // splits a lane polls in one round (all loads in flight together)
        const DevBuf bc = dev_buf(mg.cells);
        const int d = threadIdx.x % HD, sp0 = threadIdx.x / HD;
        for (int rr = n_splits - 1 - split; rr < R; rr += n_splits) {
            const int m = m_first + rr % q_len, head = kvh * G + rr / q_len;
            const int base = ((m * H + head) * n_splits) * PC;
            float mm = -INFINITY, o = 0.f, l = 0.f;
            for (int s0 = sp0; s0 < n_splits; s0 += MU * P) {
                u32x2 co[MU];
                u32x4 cml[MU];
                unsigned spins = 0;
                while (true) {
                    asm volatile("" ::: "memory");      // the cells change under our feet: every round reads memory again
                    bool ok = true;
#pragma unroll
                    for (int u = 0; u < MU; ++u) {
                        const int sp = min(s0 + u * P, n_splits - 1);       // past the end: the last split again, ignored below
                        co[u] = ld_cell1(bc, base + sp * PC + d);
                        cml[u] = ld_cells2(bc, base + sp * PC + HD);
                    }
#pragma unroll
                    for (int u = 0; u < MU; ++u) ok = ok && co[u].y == mg.flag && cml[u].y == mg.flag && cml[u].w == mg.flag;
                    if (ok) break;
                    if (++spins > mg.spin_limit) { atomicOr(mg.status, 16); break; }
                }
                float gm = mm;
#pragma unroll
                for (int u = 0; u < MU; ++u)
                    if (s0 + u * P < n_splits) gm = fmaxf(gm, __uint_as_float(cml[u].x));
                if (gm == -INFINITY) continue;
                const float keep = __expf(mm - gm);     // 0 when nothing was accumulated yet
                o *= keep; l *= keep;
#pragma unroll
                for (int u = 0; u < MU; ++u) {
                    const float mv = __uint_as_float(cml[u].x);
                    if (s0 + u * P >= n_splits || mv == -INFINITY) continue;
                    const float f = __expf(mv - gm);
                    l += __uint_as_float(cml[u].z) * f;
                    o += __uint_as_float(co[u].x) * f;
                }
                mm = gm;
            }
            __syncthreads();                         // wo / wm / wl are free again
            wo[sp0][0][d] = o;
            if (d == 0) { wm[sp0][0] = mm; wl[sp0][0] = l; }
            __syncthreads();
            if (sp0 == 0) {
                float gm = wm[0][0];
#pragma unroll
                for (int p = 1; p < P; ++p) gm = fmaxf(gm, wm[p][0]);
                float ov = 0.f, lv = 0.f;
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const float f = (wm[p][0] == -INFINITY) ? 0.f : __expf(wm[p][0] - gm);
                    ov += wo[p][0][d] * f;
                    lv += wl[p][0] * f;
                }
                Act<uint16_t>::store(mg.out, mg.plane, mg.tiled ? xt_index(m, head * HD + d) : ((size_t)m * H + head) * HD + d,
                                     lv > 0.f ? ov / lv : 0.f);
            }
        }
    }
}

// grid (M*H), threads hd: combine the splits, normalise, store in the storage dtype.  One pass: the (max, sum, o) of
// 16 splits are requested together and folded into a running (max, sum, o) -- the partials were written by other dies
// a moment ago, so every dependent round of loads is a trip to memory.
template <typename T>
__global__ void attn_merge_kernel(const float* __restrict__ part, int n_splits, int hd, size_t plane, void* __restrict__ out, int tiled_H) {
    const size_t mh = blockIdx.x;
    const int d = threadIdx.x;
    const size_t pstride = (size_t)hd + 4;       // o[hd], max, sum, 2 pad: rows stay 16-byte aligned
    const float* base = part + mh * n_splits * pstride;
    float mm = -INFINITY, o = 0.f, l = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += 16) {
        float mv[16], lv[16], ov[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const float* ps = base + (size_t)min(s0 + u, n_splits - 1) * pstride;
            mv[u] = ps[hd]; lv[u] = ps[hd + 1]; ov[u] = ps[d];
            if (s0 + u >= n_splits) mv[u] = -INFINITY;
        }
        float gm = mm;
#pragma unroll
        for (int u = 0; u < 16; ++u) gm = fmaxf(gm, mv[u]);
        if (gm == -INFINITY) continue;
        const float keep = __expf(mm - gm);       // 0 when nothing was accumulated yet
        o *= keep; l *= keep;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const float f = (mv[u] == -INFINITY) ? 0.f : __expf(mv[u] - gm);
            if (f == 0.f) continue;               // an empty split's o[] was never written
            l += lv[u] * f;
            o += ov[u] * f;
        }
        mm = gm;
    }
    // tiled_H > 0: planes in the layout of the whole-K projections (xt_index), row = mh / H, column = (mh % H) * hd + d
    const size_t idx = tiled_H > 0 ? xt_index((int)(mh / tiled_H), (int)(mh % tiled_H) * hd + d) : mh * hd + d;
    Act<T>::store(out, plane, idx, l > 0.f ? o / l : 0.f);
}

// ---- launchers -----------------------------------------------------------------------------------
int launch_prep(const int32_t* q_tokens, int q_stride, const int32_t* kv_len, int kv_base, int B, int q_len,
                int max_len, int V, int hd, float rope_base, int32_t* pos, int32_t* tok, float2* rope,
                int32_t* status, void* clear, size_t clear_bytes, hipStream_t s) {
    const int threads = q_len > 16 ? 1024 : 128;
    const size_t clear16 = clear_bytes / 16;
    // one clearing block per 32 KiB, at most 512 (a few MB of attention cells: two or three sweeps per lane)
    int extra = (int)((clear_bytes + 32767) / 32768);
    if (extra > 512) extra = 512;
    hipLaunchKernelGGL(prep_kernel, dim3(B + extra), dim3(threads), 0, s, q_tokens, q_stride, kv_len, kv_base, q_len, max_len, V,
                       hd / 2, rope_base, pos, tok, rope, status, B, reinterpret_cast<uint4*>(clear), clear16);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_embed_dec(const int32_t* tok, const void* embed, const float* gain, int M, int d, float* x, void* planes,
                     size_t plane, float* ssq, hipStream_t s) {
    hipLaunchKernelGGL(embed_dec_kernel, dim3(M), dim3(256), 0, s, tok, (const uint16_t*)embed, gain, d, x, (uint16_t*)planes, plane, ssq);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

// LDS the fused few-row projection needs for its activations; it fits next to the 8 KiB reduction buffer
// inside the 64 KiB a workgroup may use.
static size_t dec_lds_bytes(int M, int K) { return (size_t)2 * M * (K + 8) * 2; }
bool gemm_dec_fits(int M, int K) { return M >= 1 && M <= DEC_MAX_ROWS && K % 32 == 0 && dec_lds_bytes(M, K) <= 56 * 1024; }

int launch_gemm_dec(int epi, const DecArgs& a, hipStream_t s) {
    BS_REQUIRE(gemm_dec_fits(a.M, a.K), BS_ESHAPE, "gemm_dec: %d rows x %d columns of activations do not fit LDS", a.M, a.K);
    BS_REQUIRE(a.M >= 1 && a.M <= 16 && a.K % 32 == 0 && a.N % 16 == 0 && a.K >= 32, BS_ESHAPE, "gemm_dec: M=%d N=%d K=%d", a.M, a.N, a.K);
    BS_REQUIRE((double)a.N * a.K * 2.0 < 4294967296.0 && (double)a.M * a.K * 2.0 < 4294967296.0, BS_ESHAPE,
               "gemm_dec: a matrix of %d x %d exceeds the 32-bit byte offsets of this kernel", a.N, a.K);
    BS_REQUIRE(!a.att_part || (epi == EPI_RESID && a.att_splits >= 1 && (a.hd == 64 || a.hd == 128) && a.K == a.H * a.hd), BS_ESHAPE,
               "gemm_dec: attention partials as input need the O projection's shape (K = %d, H = %d, hd = %d)", a.K, a.H, a.hd);
    BS_REQUIRE(epi != EPI_QKV || (a.hd % 16 == 0 && a.seg_rows[0] % 16 == 0 && a.seg_rows[1] % 16 == 0), BS_ESHAPE, "gemm_dec: head_dim %d", a.hd);
    const int steps = a.K / 32;
    // wavefronts per 16-column tile: about six k steps each, 4 or 8 of them; the gate/up pair takes 4 + 4
    int W = (epi == EPI_SWIGLU) ? 8 : (steps >= 48 ? 8 : 4);
    const bool deep = steps / (epi == EPI_SWIGLU ? 4 : W) > 4;      // ring of 8 unless a wavefront has at most 4 steps
    const dim3 grid(a.N / 16), block(64 * W);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    { const int prc = prof_events(s, &e0, &e1); if (prc != BS_OK) return prc; }
    const size_t lds = dec_lds_bytes(a.M, a.K);
#define BS_DEC(E, MG) do { if (deep) BS_LAUNCH_TIMED((gemm_dec_kernel<E, 8, MG>), grid, block, lds, s, e0, e1, a); \
                           else BS_LAUNCH_TIMED((gemm_dec_kernel<E, 4, MG>), grid, block, lds, s, e0, e1, a); } while (0)
    if (epi == EPI_RESID && a.att_part) BS_DEC(EPI_RESID, true);
    else if (epi == EPI_RESID) BS_DEC(EPI_RESID, false);
    else if (epi == EPI_QKV) BS_DEC(EPI_QKV, false);
    else BS_DEC(EPI_SWIGLU, false);
#undef BS_DEC
    BS_LAUNCH_CHECK();
    prof_record(e0, e1, (double)a.N * (double)a.K * 2.0 * (epi == EPI_SWIGLU ? 2.0 : 1.0), 50);   // class 50: fused few-row projections
    return BS_OK;
}

// The fused projections for up to 16 rows: how many units (16-column tiles of the stacked QKV matrices; gate/up pairs)
// a workgroup gets at most, 0 when the kernel does not apply.  *grid: workgroups (one per compute unit at most).
int gemm_rows_units(int epi, int M, int N, int K, int* grid) {
    if (epi != EPI_QKV && epi != EPI_SWIGLU && epi != EPI_RESID) return 0;
    if (M < 1 || M > 16 || K < 32 || K % 32 != 0 || N < 16 || N % 16 != 0) return 0;
    if ((double)N * K * 2.0 >= 4294967296.0 || (double)M * K * 2.0 >= 4294967296.0) return 0;
    const int cus = step_grid();
    if (cus < 8) return 0;
    const int units = N / 16, G = units < cus ? units : cus;
    const int tu = (units + G - 1) / G;
    if (tu > (epi == EPI_SWIGLU ? ROWS_UMAX - 1 : ROWS_UMAX)) return 0;       // 8 KB of LDS per tile and workgroup, 64 KB at most
    if (grid) *grid = G;
    return tu;
}

int launch_gemm_rows(int epi, const DecArgs& a, hipStream_t s) {
    int G = 0;
    const int tu = gemm_rows_units(epi, a.M, a.N, a.K, &G);
    BS_REQUIRE(tu >= 1, BS_ESHAPE, "gemm_rows: M=%d N=%d K=%d", a.M, a.N, a.K);
    BS_REQUIRE(epi != EPI_QKV || ((a.hd == 64 || a.hd == 128) && a.seg_rows[0] % 16 == 0 && a.seg_rows[1] % 16 == 0 && a.q_len >= 1), BS_ESHAPE,
               "gemm_rows: head_dim %d", a.hd);
    BS_REQUIRE(epi == EPI_RESID || (a.ssq_in && a.ssq_tiles >= 1), BS_EINVAL, "gemm_rows: the input rows' sums of squares are missing");
    BS_REQUIRE(epi != EPI_RESID || (a.x && (!a.gain_next || a.out_planes)), BS_EINVAL, "gemm_rows: residual or output planes missing");
    BS_REQUIRE(epi != EPI_SWIGLU || (a.out_planes && a.w[0] && a.w[1]), BS_EINVAL, "gemm_rows: gate/up matrices or output planes missing");
    BS_REQUIRE(epi != EPI_QKV || (a.q_out && a.k_cache && a.v_cache && a.pos && a.rope), BS_EINVAL, "gemm_rows: QKV outputs or positions missing");
    BS_REQUIRE(a.xh && a.w[0], BS_EINVAL, "gemm_rows: input planes or weights missing");
    const int units = a.N / 16;
    const dim3 grid(G), block(512);
    const size_t lds = ((size_t)8 * tu * (epi == EPI_SWIGLU ? 2 : 1) * 256 + 8 * 16) * sizeof(float);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    { const int prc = prof_events(s, &e0, &e1); if (prc != BS_OK) return prc; }
#define BS_ROWS(E) do { switch (tu) { \
        case 1: BS_LAUNCH_TIMED((gemm_rows_kernel<E, 1>), grid, block, lds, s, e0, e1, a, units); break; \
        case 2: BS_LAUNCH_TIMED((gemm_rows_kernel<E, 2>), grid, block, lds, s, e0, e1, a, units); break; \
        case 3: BS_LAUNCH_TIMED((gemm_rows_kernel<E, 3>), grid, block, lds, s, e0, e1, a, units); break; \
        default: BS_LAUNCH_TIMED((gemm_rows_kernel<E, 4>), grid, block, lds, s, e0, e1, a, units); break; } } while (0)
    if (epi == EPI_QKV) BS_ROWS(EPI_QKV); else if (epi == EPI_SWIGLU) BS_ROWS(EPI_SWIGLU); else BS_ROWS(EPI_RESID);
#undef BS_ROWS
    BS_LAUNCH_CHECK();
    prof_record(e0, e1, (double)a.N * (double)a.K * 2.0 * (epi == EPI_SWIGLU ? 2.0 : 1.0), 60);   // class 60: fused projections, up to 16 rows
    return BS_OK;
}

int norm_chunks(int d) { return (d + 1023) / 1024; }

int launch_embed(int dtype, const int32_t* tok, const void* embed, int M, int d, float* x, hipStream_t s) {
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((embed_kernel<uint16_t>), dim3(M), dim3(256), 0, s, tok, (const uint16_t*)embed, d, x);
    else
        hipLaunchKernelGGL((embed_kernel<float>), dim3(M), dim3(256), 0, s, tok, (const float*)embed, d, x);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_rmsnorm(int dtype, float* x, const float* pend, int pend_ks, size_t pend_stride, const float* gain, int d,
                   float eps, int n_seq, int rows_in, int rows_out, size_t plane, void* out, hipStream_t s) {
    const int rows = n_seq * rows_out;
    if (rows <= 0) return BS_OK;
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((rmsnorm_kernel<uint16_t>), dim3(rows), dim3(1024), 0, s, x, pend, pend_ks, pend_stride, gain, d, eps, rows_in, rows_out, plane, out);
    else
        hipLaunchKernelGGL((rmsnorm_kernel<float>), dim3(rows), dim3(1024), 0, s, x, pend, pend_ks, pend_stride, gain, d, eps, rows_in, rows_out, plane, out);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_resid_sum(float* x, const float* pend, int pend_ks, size_t pend_stride, const float* gain, int d, int rows,
                     size_t plane, void* out, float* ssq, bool tiled, hipStream_t s) {
    if (rows <= 0) return BS_OK;
    BS_REQUIRE(!tiled || (rows <= 16 && d % 32 == 0), BS_ESHAPE, "resid_sum: tiled planes hold at most 16 rows (%d) of a multiple of 32 columns (%d)", rows, d);
    hipLaunchKernelGGL(resid_sum_kernel, dim3(rows, norm_chunks(d)), dim3(256), 0, s, x, pend, pend_ks, pend_stride, gain, d, plane,
                       (uint16_t*)out, ssq, tiled ? 1 : 0);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_swiglu(int dtype, const float* part, int ks, size_t ks_stride, int M, int ff, size_t plane, void* out,
                  const float* ssq, int d, float eps, hipStream_t s) {
    const size_t n = (size_t)M * ff;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    const int nch = norm_chunks(d);
    const float inv_d = 1.0f / (float)d;
    if (dtype == BS_BF16) hipLaunchKernelGGL((swiglu_kernel<uint16_t>), grid, block, 0, s, part, ks, ks_stride, M, ff, plane, out, ssq, nch, inv_d, eps);
    else hipLaunchKernelGGL((swiglu_kernel<float>), grid, block, 0, s, part, ks, ks_stride, M, ff, plane, out, ssq, nch, inv_d, eps);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

int launch_rope_kv(int dtype, const float* part, int ks, size_t ks_stride, const int32_t* pos, const float2* rope, int M,
                   int q_len, int H, int KVH, int hd, int max_len, float* q_out, void* k_cache, void* v_cache,
                   const float* ssq, int d, float eps, hipStream_t s) {
    const dim3 grid(M, H + 2 * KVH), block(hd / 2);
    const int nch = norm_chunks(d);
    const float inv_d = 1.0f / (float)d;
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((rope_kv_kernel<uint16_t>), grid, block, 0, s, part, ks, ks_stride, pos, rope, q_len, H, KVH, hd,
                           max_len, q_out, (uint16_t*)k_cache, (uint16_t*)v_cache, ssq, nch, inv_d, eps);
    else
        hipLaunchKernelGGL((rope_kv_kernel<float>), grid, block, 0, s, part, ks, ks_stride, pos, rope, q_len, H, KVH, hd,
                           max_len, q_out, (float*)k_cache, (float*)v_cache, ssq, nch, inv_d, eps);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

// bytes of the exchange cells through which the key splits of `rows` query rows are combined inside the attention kernel
size_t attn_cells_bytes(int rows, int H, int hd, int n_splits) {
    const double b = (double)rows * H * n_splits * (hd + 4) * 8.0;
    return b < 2147483648.0 ? (size_t)b : 0;           // 32-bit cell offsets
}

// workgroups of the one-tile attention kernel that the device holds at the same time
static size_t attn_resident_workgroups(int hd) {
    auto ask = [](bool wide) -> size_t {
        int per_cu = 0;
        const hipError_t e = wide ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_mfma_kernel<128, 1>, 256, 0)
                                  : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_mfma_kernel<64, 1>, 256, 0);
        const int cus = step_grid();
        return (e == hipSuccess && per_cu > 0 && cus > 0) ? (size_t)per_cu * cus : 1;   // 1: never enough, the merge kernel runs
    };
    static const size_t c128 = ask(true), c64 = ask(false);      // asked once (initialisation of a local static is thread-safe)
    return hd == 128 ? c128 : c64;
}

int launch_attention(int dtype, const float* q, const void* k_cache, const void* v_cache, const int32_t* pos, int B,
                     int q_len, int H, int KVH, int hd, int max_len, int n_splits, float* part, size_t plane, void* out,
                     bool out_tiled, const AttnCells* cells, hipStream_t s) {
    BS_REQUIRE(!out_tiled || (dtype == BS_BF16 && out && n_splits > 1 && B * q_len <= 16), BS_ESHAPE,
               "attention: tiled output planes are written by the merge of several key splits of at most 16 rows");
    const float scale = 1.0f / sqrtf((float)hd);
    const dim3 grid(n_splits, H, B), block(256);
    if (dtype == BS_BF16) {
        // Many query rows per head group (prompt chunks): one workgroup per group of row tiles and only as many key
        // splits as it takes to reach about a thousand workgroups; a single group keeps all the splits.
        const int n_tiles = (H / KVH * q_len + 15) / 16;
        // two tiles per wavefront as soon as there are two: a K or V block then serves 32 rows (verification with grouped
        // queries: 287 -> 225 us per layer at batch 32 / 8192 keys; prompt chunks of a batch: 7-10 % off the prompt pass)
        const int nt = (n_tiles >= 2) ? 2 : 1;
        const int n_rt = (n_tiles + nt - 1) / nt;
        if (out && n_rt > 1) {
            const int want = (1024 + B * KVH * n_rt - 1) / (B * KVH * n_rt);
            n_splits = want < n_splits ? want : n_splits;
        }
        const dim3 mgrid(n_splits * (out ? n_rt : 1), KVH, B);
        uint16_t* direct = (out && n_splits == 1) ? reinterpret_cast<uint16_t*>(out) : nullptr;     // no merge needed
        // the splits combined inside the kernel: one row tile, exchange cells at hand, every workgroup resident at once
        AttnMerge mg = {};
        if (cells && cells->buf && out && !direct && nt == 1 && n_rt == 1 && attn_cells_bytes(B * q_len, H, hd, n_splits) <= cells->bytes &&
            (size_t)n_splits * KVH * B <= attn_resident_workgroups(hd)) {
            mg.cells = cells->buf; mg.out = reinterpret_cast<uint16_t*>(out); mg.plane = plane; mg.tiled = out_tiled ? 1 : 0;
            mg.flag = cells->flag; mg.spin_limit = cells->spin_limit; mg.status = cells->status;
        }
        hipEvent_t e0 = nullptr, e1 = nullptr;
        { const int prc = prof_events(s, &e0, &e1); if (prc != BS_OK) return prc; }
#define BS_ATTN(HD, NT) BS_LAUNCH_TIMED((attn_mfma_kernel<HD, NT>), mgrid, block, 0, s, e0, e1, q, (const uint16_t*)k_cache, \
                                        (const uint16_t*)v_cache, pos, q_len, H, KVH, max_len, scale, part, n_splits, direct, plane, mg)
        if (hd == 128) { if (nt == 2) BS_ATTN(128, 2); else BS_ATTN(128, 1); }
        else if (hd == 64) { if (nt == 2) BS_ATTN(64, 2); else BS_ATTN(64, 1); }
        else
            BS_FAIL(BS_ESHAPE, "attention: bf16 caches need head_dim 64 or 128, got %d", hd);
#undef BS_ATTN
        BS_LAUNCH_CHECK();
        prof_record(e0, e1, 0.0, 100);                     // class 100: the split attention kernel (bytes known to the caller)
        if (out && !direct && !mg.cells) hipLaunchKernelGGL((attn_merge_kernel<uint16_t>), dim3(B * q_len * H), dim3(hd), 0, s, part, n_splits, hd, plane, out, out_tiled ? H : 0);
    } else {
        hipLaunchKernelGGL((attn_kernel<float>), grid, block, 0, s, q, (const float*)k_cache,
                           (const float*)v_cache, pos, q_len, H, KVH, hd, max_len, scale, part);
        BS_LAUNCH_CHECK();
        hipLaunchKernelGGL((attn_merge_kernel<float>), dim3(B * q_len * H), dim3(hd), 0, s, part, n_splits, hd, plane, out, out_tiled ? H : 0);
    }
    BS_LAUNCH_CHECK();
    return BS_OK;
}

}  // namespace bs
