// Vocabulary-wide softmax + accept/reject + residual/bonus sampling (App. A, vanilla speculative
// decoding: the loop over draft positions and the bonus draw), and the categorical draw used by
// the draft steps.
//
// Two kernels.  Phase A streams every logit row once (one workgroup per row) and leaves its softmax
// statistics (max, sum of exp): this is the HBM-bound part, about 2 exponentials per logit.  Phase B runs
// one workgroup per sequence: the gamma acceptance tests u * q(x~) <= p(x~) need only those statistics and
// two logits each; the first failure fixes the deciding position, and only that row pair is read again
// (from cache, it was just streamed) and sampled: from [p - q]_+ if a draft token was rejected, from p at the
// bonus position otherwise.  (The draft draw of a single short row keeps the row in registers instead.)  The sequential
// accept chain of the algorithm costs gamma scalar tests; the vocabulary-wide work is parallel.
//
// Reductions: per-lane online softmax (max, sum) -> wavefront shuffles -> LDS across 8 wavefronts.
// Inverse CDF in increasing token id: lane t owns 8-token groups t, t+512, ...; "slab" k is the
// 4096 consecutive tokens of groups [512k, 512k+512).  Slab totals locate the slab, a block-wide
// scan of the 512 group sums locates the group, a serial scan of 8 weights locates the token.
#include <math.h>
#include <mutex>
#include "common.h"
#include "sample.h"

namespace bs {

constexpr int ST = 512;           // lanes per workgroup
constexpr int SW = ST / 64;       // wavefronts per workgroup
constexpr int GE = 8;             // tokens per group
constexpr int MAX_SLABS = 256;    // V <= 2^20
constexpr int SLAB_BATCH = 4;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// A group = tokens [8g, 8g+8) of a row, held as loaded (16 B of bf16, or 32 B of float); tokens >= V
// read as -inf.  expand() turns it into floats scaled by 1/temperature.
template <typename T> struct Raw;
template <> struct Raw<uint16_t> { uint4 v; };
template <> struct Raw<float> { float4 a, b; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ Raw<uint16_t> neg_inf_raw(const uint16_t*) {
    Raw<uint16_t> r; r.v = make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u); return r;
}
__device__ __forceinline__ Raw<float> neg_inf_raw(const float*) {
    Raw<float> r; r.a = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY); r.b = r.a; return r;
}

__device__ __forceinline__ Raw<uint16_t> load_raw_vec(const uint16_t* __restrict__ row, int g) {
    Raw<uint16_t> r;
    r.v = *reinterpret_cast<const uint4*>(row + g * GE);
    return r;
}
__device__ __forceinline__ Raw<float> load_raw_vec(const float* __restrict__ row, int g) {
    Raw<float> r;
    r.a = *reinterpret_cast<const float4*>(row + g * GE);
    r.b = *reinterpret_cast<const float4*>(row + g * GE + 4);
    return r;
}
__device__ __forceinline__ Raw<uint16_t> load_raw(const uint16_t* __restrict__ row, int g, int V, bool vec_ok) {
    const int base = g * GE;
    Raw<uint16_t> r;
    if (vec_ok && base + GE <= V) {
        r.v = *reinterpret_cast<const uint4*>(row + base);
    } else {
        uint32_t h[GE];
#pragma unroll
        for (int e = 0; e < GE; ++e) h[e] = (base + e < V) ? (uint32_t)row[base + e] : 0xFF80u;
        r.v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
    return r;
}
__device__ __forceinline__ Raw<float> load_raw(const float* __restrict__ row, int g, int V, bool vec_ok) {
    const int base = g * GE;
    Raw<float> r;
    if (vec_ok && base + GE <= V) {
        r.a = *reinterpret_cast<const float4*>(row + base);
        r.b = *reinterpret_cast<const float4*>(row + base + 4);
    } else {
        float h[GE];
#pragma unroll
        for (int e = 0; e < GE; ++e) h[e] = (base + e < V) ? row[base + e] : -INFINITY;
        r.a = make_float4(h[0], h[1], h[2], h[3]);
        r.b = make_float4(h[4], h[5], h[6], h[7]);
    }
    return r;
}
// Stops the compiler from carrying values derived from a group across passes.
__device__ __forceinline__ void keep_opaque(Raw<uint16_t>& r) {
    asm volatile("" : "+v"(r.v.x), "+v"(r.v.y), "+v"(r.v.z), "+v"(r.v.w));
}
__device__ __forceinline__ void keep_opaque(Raw<float>& r) {
    asm volatile("" : "+v"(r.a.x), "+v"(r.a.y), "+v"(r.a.z), "+v"(r.a.w), "+v"(r.b.x), "+v"(r.b.y), "+v"(r.b.z), "+v"(r.b.w));
}
__device__ __forceinline__ void expand(const Raw<uint16_t>& r, float s, float out[GE]) {
    out[0] = bf16_lo(r.v.x) * s; out[1] = bf16_hi(r.v.x) * s; out[2] = bf16_lo(r.v.y) * s; out[3] = bf16_hi(r.v.y) * s;
    out[4] = bf16_lo(r.v.z) * s; out[5] = bf16_hi(r.v.z) * s; out[6] = bf16_lo(r.v.w) * s; out[7] = bf16_hi(r.v.w) * s;
}
__device__ __forceinline__ void expand(const Raw<float>& r, float s, float out[GE]) {
    out[0] = r.a.x * s; out[1] = r.a.y * s; out[2] = r.a.z * s; out[3] = r.a.w * s;
    out[4] = r.b.x * s; out[5] = r.b.y * s; out[6] = r.b.z * s; out[7] = r.b.w * s;
}

template <typename T>
__device__ __forceinline__ float load_one(const T* row, int idx);
template <>
__device__ __forceinline__ float load_one<float>(const float* row, int idx) { return row[idx]; }
template <>
__device__ __forceinline__ float load_one<uint16_t>(const uint16_t* row, int idx) {
    return __uint_as_float((uint32_t)row[idx] << 16);
}

struct RowShared {
    float red[4][SW];                 // also the staging of SLAB_BATCH slab sums
    float slab_tot[MAX_SLABS];
    float wave_tot[SW];
    int wave_first[SW];
    int wave_last[SW];
    float bcast[8];
    int ibcast[4];
};

static_assert(SLAB_BATCH <= 4, "RowShared::red has four rows");

struct RowResult {
    int token;        // candidate token of this row (valid in every lane)
    float p_x, q_x;   // normalised probabilities of the drafted token (lane 0 only, if x >= 0)
    int fallback;     // residual had no mass: drew from p instead
};

// Processes one row pair.  has_q = false: the draw is from softmax(p) (bonus token, draft draws).
// x = drafted token for the acceptance test, or -1.
template <typename T, int NG, bool CACHED>
__device__ RowResult process_row(const T* __restrict__ p, const T* __restrict__ q, bool has_q, int V, float inv_temp,
                                 int x, float u_final, RowShared& sh, const float* known = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int ngroups = (V + GE - 1) / GE;
    const int nslabs = (ngroups + ST - 1) / ST;
    const bool vec_p = ((reinterpret_cast<uintptr_t>(p) & 15) == 0);
    const bool vec_q = has_q && ((reinterpret_cast<uintptr_t>(q) & 15) == 0);

    Raw<T> pv[CACHED ? NG : 1], qv[CACHED ? NG : 1];

    // ---- pass 1: the only HBM read; per-lane online (max, sum of exp) for both rows ----
    float mp = -INFINITY, sp = 0.f, mq = -INFINITY, sq = 0.f;
    auto online = [&](float& m, float& s, const Raw<T>& raw) {
        float v[GE];
        expand(raw, inv_temp, v);
        float gm = v[0];
#pragma unroll
        for (int e = 1; e < GE; ++e) gm = fmaxf(gm, v[e]);
        if (gm == -INFINITY) return;
        const float mn = fmaxf(m, gm);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < GE; ++e) acc += __expf(v[e] - mn);
        s = s * __expf(m - mn) + acc;
        m = mn;
    };
    if constexpr (CACHED) {
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            const int g = tid + k * ST;
            // the host launches this variant only for 16-byte aligned rows with V % 8 == 0
            pv[k] = (g < ngroups) ? load_raw_vec(p, g) : neg_inf_raw(p);
            qv[k] = (has_q && g < ngroups) ? load_raw_vec(q, g) : neg_inf_raw(p);
        }
        if (!known) {
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                online(mp, sp, pv[k]);
                if (has_q) online(mq, sq, qv[k]);
                __builtin_amdgcn_sched_barrier(0);   // one group at a time: keeps the live set small
            }
        }
    } else if (!known) {
        for (int g = tid; g < ngroups; g += ST) {
            online(mp, sp, load_raw(p, g, V, vec_p));
            if (has_q) online(mq, sq, load_raw(q, g, V, vec_q));
        }
    }
    if constexpr (CACHED) {
        // the later passes recompute from the packed registers instead of keeping expanded values alive
#pragma unroll
        for (int k = 0; k < NG; ++k) { keep_opaque(pv[k]); keep_opaque(qv[k]); }
    }
    // block combine of (max, sum): maxima first, then rescaled sums (skipped when the row statistics are given)
    if (known) {
        mp = known[0]; sp = known[1]; mq = known[2]; sq = known[3];
    } else {
        const float wmp = wave_max(mp), wmq = wave_max(mq);
        if (lane == 0) { sh.red[0][wid] = wmp; sh.red[1][wid] = wmq; }
        __syncthreads();
        float bmp = sh.red[0][0], bmq = sh.red[1][0];
#pragma unroll
        for (int w = 1; w < SW; ++w) { bmp = fmaxf(bmp, sh.red[0][w]); bmq = fmaxf(bmq, sh.red[1][w]); }
        const float rp = (mp == -INFINITY) ? 0.f : sp * __expf(mp - bmp);
        const float rq = (mq == -INFINITY) ? 0.f : sq * __expf(mq - bmq);
        const float wsp = wave_sum(rp), wsq = wave_sum(rq);
        if (lane == 0) { sh.red[2][wid] = wsp; sh.red[3][wid] = wsq; }
        __syncthreads();
        float zp = 0.f, zq = 0.f;
#pragma unroll
        for (int w = 0; w < SW; ++w) { zp += sh.red[2][w]; zq += sh.red[3][w]; }
        mp = bmp; mq = bmq; sp = zp; sq = zq;
    }
    const float inv_zp = 1.0f / sp;
    const float inv_zq = has_q ? 1.0f / sq : 0.f;

    RowResult res;
    res.p_x = 0.f; res.q_x = 0.f; res.fallback = 0; res.token = 0;
    if (tid == 0 && x >= 0) {
        res.p_x = __expf(load_one<T>(p, x) * inv_temp - mp) * inv_zp;
        res.q_x = has_q ? __expf(load_one<T>(q, x) * inv_temp - mq) * inv_zq : 0.f;
    }

    // ---- weights of the draw: [p - q]_+ (normalised probabilities) or exp(p - max) ----
    bool residual = has_q;
    auto weights = [&](const Raw<T>& ra, const Raw<T>& rb, float w[GE]) {
        float a[GE];
        expand(ra, inv_temp, a);
        if (residual) {
            float b[GE];
            expand(rb, inv_temp, b);
#pragma unroll
            for (int e = 0; e < GE; ++e)
                w[e] = fmaxf(__expf(a[e] - mp) * inv_zp - __expf(b[e] - mq) * inv_zq, 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < GE; ++e) w[e] = __expf(a[e] - mp);
        }
    };
    auto group_weights = [&](int k, int g, float w[GE]) {
        if (g >= ngroups) {
#pragma unroll
            for (int e = 0; e < GE; ++e) w[e] = 0.f;
            return;
        }
        if constexpr (CACHED) {
            weights(pv[k], qv[k], w);
        } else {
            const Raw<T> ra = load_raw(p, g, V, vec_p);
            const Raw<T> rb = residual ? load_raw(q, g, V, vec_q) : ra;
            weights(ra, rb, w);
        }
    };
    auto group_sum = [&](int k, int g) {
        float w[GE];
        group_weights(k, g, w);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < GE; ++e) s += w[e];
        return s;
    };

    float total = 0.f;
#pragma nounroll
    for (int attempt = 0; attempt < 2; ++attempt) {
        // ---- pass 2: slab totals ----
        if constexpr (CACHED) {
            float ss[NG];
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                ss[k] = group_sum(k, tid + k * ST);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int k = 0; k < NG; ++k) ss[k] = wave_sum(ss[k]);
            __syncthreads();
            if (lane == 0) {
#pragma unroll
                for (int k = 0; k < NG; ++k) sh.slab_tot[k * SW + wid] = ss[k];   // staging: [slab][wave]
            }
            __syncthreads();
            float tot[NG];
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                float t = 0.f;
#pragma unroll
                for (int w = 0; w < SW; ++w) t += sh.slab_tot[k * SW + w];
                tot[k] = t;
            }
            __syncthreads();
            if (tid == 0) {
#pragma unroll
                for (int k = 0; k < NG; ++k) sh.slab_tot[k] = tot[k];
            }
            __syncthreads();
        } else {
            for (int k0 = 0; k0 < nslabs; k0 += SLAB_BATCH) {
                float ss[SLAB_BATCH];
#pragma unroll
                for (int j = 0; j < SLAB_BATCH; ++j)
                    ss[j] = (k0 + j < nslabs) ? wave_sum(group_sum(k0 + j, tid + (k0 + j) * ST)) : 0.f;
                __syncthreads();
                if (lane == 0) {
#pragma unroll
                    for (int j = 0; j < SLAB_BATCH; ++j) sh.red[j][wid] = ss[j];
                }
                __syncthreads();
                if (tid < SLAB_BATCH && k0 + tid < nslabs) {
                    float t = 0.f;
#pragma unroll
                    for (int w = 0; w < SW; ++w) t += sh.red[tid][w];
                    sh.slab_tot[k0 + tid] = t;
                }
            }
            __syncthreads();
        }
        total = 0.f;
        for (int k = 0; k < nslabs; ++k) total += sh.slab_tot[k];
        if (!residual || total > 0.f) break;
        // residual without mass (p == q up to rounding): draw from p instead
        residual = false;
        res.fallback = 1;
        __syncthreads();
    }

    // ---- locate the slab ----
    const float thr = u_final * total;
    int kstar = -1;
    float base = 0.f;
    {
        float run = 0.f;
        int last_pos = 0;
        float last_base = 0.f;
        for (int k = 0; k < nslabs; ++k) {
            const float t = sh.slab_tot[k];
            if (t > 0.f) { last_pos = k; last_base = run; }
            if (run + t > thr) { kstar = k; base = run; break; }
            run += t;
        }
        if (kstar < 0) { kstar = last_pos; base = last_base; }   // thr >= total only through rounding
    }

    // ---- pass 3: scan of the 1024 group sums of slab kstar ----
    float w[GE];
    {
        const int g = tid + kstar * ST;
        if constexpr (CACHED) {
            // select the register slab without dynamic indexing, then recompute its weights (cheaper
            // in registers than keeping every slab's weights alive since pass 2)
#pragma unroll
            for (int k = 0; k < NG; ++k) { keep_opaque(pv[k]); keep_opaque(qv[k]); }
            Raw<T> sp_ = pv[0], sq_ = qv[0];
#pragma unroll
            for (int k = 1; k < NG; ++k) {
                if (k == kstar) { sp_ = pv[k]; sq_ = qv[k]; }
            }
            keep_opaque(sp_);
            keep_opaque(sq_);
            if (g < ngroups) {
                weights(sp_, sq_, w);
            } else {
#pragma unroll
                for (int e = 0; e < GE; ++e) w[e] = 0.f;
            }
        } else {
            group_weights(kstar, g, w);
        }
    }
    float gs = 0.f;
#pragma unroll
    for (int e = 0; e < GE; ++e) gs += w[e];
    float incl = gs;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    __syncthreads();
    if (lane == 63) sh.wave_tot[wid] = incl;
    __syncthreads();
    float before = base;
    for (int wv = 0; wv < wid; ++wv) before += sh.wave_tot[wv];
    incl += before;
    // The shuffled prefix is not monotone in fp32 (every lane sums in its own order), so an empty group can be the first
    // whose prefix exceeds thr: only groups that carry mass may be hit, and below only tokens that do.
    const bool hit = incl > thr && gs > 0.f;
    const uint64_t mhit = __ballot(hit);
    const uint64_t mpos = __ballot(gs > 0.f);
    if (lane == 0) {
        sh.wave_first[wid] = mhit ? (__ffsll((long long)mhit) - 1) : 64;
        sh.wave_last[wid] = mpos ? (63 - __clzll((long long)mpos)) : -1;
    }
    __syncthreads();
    int tstar = -1, tlast = -1;
    for (int wv = 0; wv < SW; ++wv) {
        if (tstar < 0 && sh.wave_first[wv] < 64) tstar = wv * 64 + sh.wave_first[wv];
        if (sh.wave_last[wv] >= 0) tlast = wv * 64 + sh.wave_last[wv];
    }
    const bool forced = tstar < 0;            // rounding pushed thr past this slab's scan total
    if (forced) tstar = tlast;
    if (tid == tstar) {
        float run = incl - gs;
        int pick = -1, lastpos = 0;
#pragma unroll
        for (int e = 0; e < GE; ++e) {
            run += w[e];
            if (w[e] > 0.f) lastpos = e;
            if (pick < 0 && !forced && run > thr && w[e] > 0.f) pick = e;
        }
        if (pick < 0) pick = lastpos;
        sh.ibcast[0] = (tid + kstar * ST) * GE + pick;
    }
    if (tstar < 0 && tid == 0) sh.ibcast[0] = 0;   // only with non-finite input
    __syncthreads();
    res.token = min(sh.ibcast[0], V - 1);
    return res;
}

// ---- phase A: softmax statistics (max, sum of exp) of every logit row, target and draft alike ----------
// One workgroup of 256 lanes per row, pure streaming: 16-byte loads, four in flight per lane, per-lane online
// (max, sum), wavefront shuffles, LDS across the 4 wavefronts.  Rows: B*(gamma+1) target rows, then B*gamma
// draft rows.  This is where the HBM bytes of the sampling step are read.
template <typename T>
__global__ __launch_bounds__(256) void row_stats_kernel(const T* __restrict__ p_logits, const T* __restrict__ q_logits,
                                                        int n_p_rows, int V, float inv_temp, float2* __restrict__ stats) {
    __shared__ float red[2][4];
    const int r = blockIdx.x;
    const T* row = r < n_p_rows ? p_logits + (size_t)r * V : q_logits + (size_t)(r - n_p_rows) * V;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int ngroups = (V + GE - 1) / GE;
    const bool vec = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    // Arithmetic per logit is what bounds this kernel as much as the bytes do (a compute unit retires 64 lane-operations
    // per cycle, and 17 rows of 32000 logits per sequence are 2100 logits per compute unit and sequence), so the inner
    // loop is kept to: widen, max (on the raw values: the scale is positive), one fused multiply-add into the base-2
    // exponent, v_exp_f32, add.  Running maximum mr in raw units; the sum is rescaled once per batch of loads.
    const float c2 = inv_temp * 1.4426950408889634f;             // logit -> base-2 exponent
    float mr = -INFINITY, sum = 0.f;
    auto raw_max = [&](const Raw<T>& raw, float cur) {
        float v[GE];
        expand(raw, 1.0f, v);
#pragma unroll
        for (int e = 0; e < GE; ++e) cur = fmaxf(cur, v[e]);
        return cur;
    };
    auto accumulate = [&](const Raw<T>& raw, float off) {       // off = -mr * c2
        float v[GE];
        expand(raw, 1.0f, v);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < GE; ++e) acc += __builtin_amdgcn_exp2f(fmaf(v[e], c2, off));
        sum += acc;
    };
    auto rebase = [&](float mn) {                               // new running maximum mn >= mr (raw units)
        if (mn > mr) {
            sum = (mr == -INFINITY) ? 0.f : sum * __builtin_amdgcn_exp2f((mr - mn) * c2);
            mr = mn;
        }
    };
    int g = tid;
    if (vec && V % GE == 0) {
        for (; g + 3 * 256 < ngroups; g += 4 * 256) {
            Raw<T> a0 = load_raw_vec(row, g), a1 = load_raw_vec(row, g + 256), a2 = load_raw_vec(row, g + 512),
                   a3 = load_raw_vec(row, g + 768);
            rebase(raw_max(a3, raw_max(a2, raw_max(a1, raw_max(a0, mr)))));
            if (mr != -INFINITY) {
                const float off = -mr * c2;
                accumulate(a0, off); accumulate(a1, off); accumulate(a2, off); accumulate(a3, off);
            }
        }
    }
    for (; g < ngroups; g += 256) {
        const Raw<T> a0 = load_raw(row, g, V, vec);
        rebase(raw_max(a0, mr));
        if (mr != -INFINITY) accumulate(a0, -mr * c2);
    }
    const float m = (mr == -INFINITY) ? -INFINITY : mr * inv_temp;     // the statistics are in natural-log units
    const float bm = wave_max(m);
    if (lane == 0) red[0][wid] = bm;
    __syncthreads();
    const float mm = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    const float rs = wave_sum(m == -INFINITY ? 0.f : sum * __expf(m - mm));
    if (lane == 0) red[1][wid] = rs;
    __syncthreads();
    if (tid == 0) stats[r] = make_float2(mm, red[1][0] + red[1][1] + red[1][2] + red[1][3]);
}

// ---- phase B: acceptance tests and the one draw each sequence needs -------------------------------------
// One workgroup per sequence.  Lanes 0..gamma-1 evaluate  u_i * q_i(x~_i) <= p_i(x~_i)  from the row statistics
// (two scalar loads each); tau = number of leading acceptances; then the workgroup re-reads only the deciding
// row pair (tau < gamma: residual [p - q]_+, else the bonus row) and draws by inverse CDF.
struct DecideParams {
    const void* p_logits;
    const void* q_logits;
    const int32_t* draft_tokens;
    const float* uniforms;
    uint64_t seed;
    const uint32_t* round_ptr;
    uint32_t round;
    int gamma, V, n_p_rows;
    float inv_temp;
    const float2* stats;
    int32_t* flags;        // [B, gamma+1] or null: bit 0 accepted, bit 1 residual fallback (at the deciding row)
    int32_t* cand;         // [B, gamma+1] or null: token written at the deciding row
    int32_t* accept_len;   // [B] or null
    int32_t* next_token;   // [B] or null
    float* margins;        // [B, gamma] or null
};

template <typename T, int NG, bool CACHED>
__global__ __launch_bounds__(ST) void spec_decide_kernel(DecideParams a) {
    __shared__ RowShared sh;
    __shared__ int s_acc[ST];
    __shared__ float2 s_sp[ST + 1], s_sq[ST];     // row statistics of this sequence: no second trip to memory for them
    __shared__ float s_known[4];
    const int b = blockIdx.x, tid = threadIdx.x, gamma = a.gamma;
    const T* P = reinterpret_cast<const T*>(a.p_logits) + (size_t)b * (gamma + 1) * a.V;
    const T* Q = reinterpret_cast<const T*>(a.q_logits) + (size_t)b * gamma * a.V;
    const uint32_t t = a.round_ptr ? *a.round_ptr : a.round;
    if (tid == 0) s_sp[gamma] = a.stats[(size_t)b * (gamma + 1) + gamma];
    for (int i = tid; i < gamma; i += ST) {
        int x = a.draft_tokens[(size_t)b * gamma + i];
        const bool okx = x >= 0 && x < a.V;
        if (!okx) x = 0;
        const float2 sp = a.stats[(size_t)b * (gamma + 1) + i], sq = a.stats[a.n_p_rows + (size_t)b * gamma + i];
        s_sp[i] = sp; s_sq[i] = sq;
        const float px = __expf(load_one<T>(P + (size_t)i * a.V, x) * a.inv_temp - sp.x) / sp.y;
        const float qx = __expf(load_one<T>(Q + (size_t)i * a.V, x) * a.inv_temp - sq.x) / sq.y;
        const float u = a.uniforms ? a.uniforms[(size_t)b * (gamma + 1) + i]
                                   : u_open_closed(philox_word(a.seed, (uint32_t)b, t, (uint32_t)i, PURPOSE_ACCEPT));
        const int acc = okx && (u * qx <= px);
        s_acc[i] = acc;
        if (a.flags) a.flags[(size_t)b * (gamma + 1) + i] = acc;
        if (a.margins) a.margins[(size_t)b * gamma + i] = okx ? ((qx > 0.f) ? fminf(1.f, px / qx) : 1.f) - u : -1.f;
    }
    __syncthreads();
    int tau = 0;
    while (tau < gamma && s_acc[tau]) ++tau;
    const bool has_q = tau < gamma;
    if (tid == 0) {
        const float2 sp = s_sp[tau];
        s_known[0] = sp.x; s_known[1] = sp.y; s_known[2] = 0.f; s_known[3] = 1.f;
        if (has_q) { const float2 sq = s_sq[tau]; s_known[2] = sq.x; s_known[3] = sq.y; }
    }
    __syncthreads();
    const float u_final = a.uniforms ? a.uniforms[(size_t)b * (gamma + 1) + gamma]
                                     : u_closed_open(philox_word(a.seed, (uint32_t)b, t, 0u, PURPOSE_FINAL));
    const RowResult r = process_row<T, NG, CACHED>(P + (size_t)tau * a.V, has_q ? Q + (size_t)tau * a.V : nullptr, has_q,
                                                   a.V, a.inv_temp, -1, u_final, sh, s_known);
    if (tid == 0) {
        if (a.flags) a.flags[(size_t)b * (gamma + 1) + tau] = (r.fallback << 1);     // bit 0 clear: not accepted / bonus row
        if (a.cand) a.cand[(size_t)b * (gamma + 1) + tau] = r.token;
        if (a.accept_len) a.accept_len[b] = tau;
        if (a.next_token) a.next_token[b] = r.token;
    }
}

// ---- greedy mode (temperature 0, Sec. 2: all mass on the largest logit) ---------------------------------
// Index of the largest logit of a row, lowest token id among equal ones.  Every lane walks its groups in
// increasing id and keeps the first strict maximum; lanes are then combined by (value desc, id asc).
struct ArgBest { float v; int i; };
__device__ __forceinline__ ArgBest better(ArgBest a, ArgBest b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
template <typename T, int NT>
__device__ __forceinline__ int block_argmax(const T* __restrict__ row, int V, ArgBest* red /* NT / 64 entries of LDS */) {
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int ngroups = (V + GE - 1) / GE;
    const bool vec = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    ArgBest best = {-INFINITY, 0x7FFFFFFF};
    for (int g = tid; g < ngroups; g += NT) {
        float v[GE];
        expand(load_raw(row, g, V, vec), 1.0f, v);
#pragma unroll
        for (int e = 0; e < GE; ++e)
            if (v[e] > best.v) { best.v = v[e]; best.i = g * GE + e; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ArgBest other;
        other.v = __shfl_xor(best.v, o, 64);
        other.i = __shfl_xor(best.i, o, 64);
        best = better(best, other);
    }
    if (lane == 0) red[wid] = best;
    __syncthreads();
    ArgBest tot = red[0];
    for (int w = 1; w < NT / 64; ++w) tot = better(tot, red[w]);
    __syncthreads();
    return tot.i < V ? tot.i : 0;                 // a row without any finite logit: token 0
}

template <typename T>
__global__ __launch_bounds__(256) void row_argmax_kernel(const T* __restrict__ rows, int V, int32_t* __restrict__ out) {
    __shared__ ArgBest red[4];
    const int k = block_argmax<T, 256>(rows + (size_t)blockIdx.x * V, V, red);
    if (threadIdx.x == 0) out[blockIdx.x] = k;
}

// one lane per sequence: tau = leading draft tokens equal to the target's argmax; the emitted token is the
// target's argmax at the first mismatch, or at the bonus position
__global__ void greedy_decide_kernel(const int32_t* __restrict__ amax, const int32_t* __restrict__ draft_tokens, int B, int gamma,
                                     int32_t* __restrict__ flags, int32_t* __restrict__ cand, int32_t* __restrict__ accept_len,
                                     int32_t* __restrict__ next_token, float* __restrict__ margins) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int tau = gamma;
    for (int i = gamma - 1; i >= 0; --i) {
        const int acc = draft_tokens[(size_t)b * gamma + i] == amax[(size_t)b * (gamma + 1) + i];
        if (!acc) tau = i;
        if (flags) flags[(size_t)b * (gamma + 1) + i] = acc;
        if (margins) margins[(size_t)b * gamma + i] = acc ? 1.f : -1.f;
    }
    const int token = amax[(size_t)b * (gamma + 1) + tau];
    if (flags) flags[(size_t)b * (gamma + 1) + tau] = 0;
    if (cand) cand[(size_t)b * (gamma + 1) + tau] = token;
    if (accept_len) accept_len[b] = tau;
    if (next_token) next_token[b] = token;
}

// Draft-step draw: x~ ~ softmax(logits[b] / T) with the Philox uniform (b, t, slot, DRAFT).
__global__ __launch_bounds__(ST) void draw_kernel(DrawParams a) {
    __shared__ RowShared sh;
    const int b = blockIdx.x;
    const float* p = a.logits + (size_t)b * a.row_stride;
    if (a.greedy) {                                  // temperature 0: the draft's argmax
        __shared__ ArgBest red[SW];
        const int k = block_argmax<float, ST>(p, a.V, red);
        if (threadIdx.x == 0) {
            if (a.out0) a.out0[(size_t)b * a.stride0 + a.off0] = k;
            if (a.out1) a.out1[(size_t)b * a.stride1 + a.off1] = k;
            if (a.out2) a.out2[(size_t)b * a.stride2 + a.off2] = k;
        }
        return;
    }
    const uint32_t t = a.round_ptr ? *a.round_ptr : a.round;
    const float u = u_closed_open(philox_word(a.seed, (uint32_t)b, t, a.slot, PURPOSE_DRAFT));
    RowResult r;
    // rows of up to 32768 logits stay in registers (eight groups per lane): one trip to memory instead of one per
    // pass over the row -- with a single sequence this kernel is one workgroup and nothing else hides its latency
    // (draft step at V = 32000: 6 us shorter)
    if (a.V <= 8 * ST * GE && a.V % GE == 0 && a.row_stride % 4 == 0 && ((uintptr_t)a.logits & 15) == 0)
        r = process_row<float, 8, true>(p, nullptr, false, a.V, a.inv_temp, -1, u, sh);
    else
        r = process_row<float, 1, false>(p, nullptr, false, a.V, a.inv_temp, -1, u, sh);
    if (threadIdx.x == 0) {
        if (a.out0) a.out0[(size_t)b * a.stride0 + a.off0] = r.token;
        if (a.out1) a.out1[(size_t)b * a.stride1 + a.off1] = r.token;
        if (a.out2) a.out2[(size_t)b * a.stride2 + a.off2] = r.token;
    }
}

int launch_draw(const DrawParams& a, int B, hipStream_t stream) {
    if (B <= 0) return BS_OK;
    hipLaunchKernelGGL(draw_kernel, dim3(B), dim3(ST), 0, stream, a);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

size_t spec_scratch_bytes(int B, int gamma) {
    return align_up((size_t)B * (2 * (size_t)gamma + 1) * sizeof(float2), 256);
}

int launch_spec_sample(const void* p_logits, const void* q_logits, const int32_t* draft_tokens, int B, int gamma, int V,
                       int dtype, float temperature, const float* uniforms, uint64_t seed, const uint32_t* round_ptr,
                       uint32_t round, void* stats_scratch, int32_t* flags, int32_t* cand, int32_t* accept_len,
                       int32_t* next_token, float* margins, hipStream_t stream) {
    if (B <= 0) return BS_OK;
    const int n_p = B * (gamma + 1), n_rows = n_p + B * gamma;
    if (temperature == 0.f) {                        // greedy: only the target rows' argmax is needed
        int32_t* amax = reinterpret_cast<int32_t*>(stats_scratch);
        if (dtype == BS_BF16) hipLaunchKernelGGL((row_argmax_kernel<uint16_t>), dim3(n_p), dim3(256), 0, stream, (const uint16_t*)p_logits, V, amax);
        else hipLaunchKernelGGL((row_argmax_kernel<float>), dim3(n_p), dim3(256), 0, stream, (const float*)p_logits, V, amax);
        BS_LAUNCH_CHECK();
        hipLaunchKernelGGL(greedy_decide_kernel, dim3((B + 127) / 128), dim3(128), 0, stream, amax, draft_tokens, B, gamma, flags, cand,
                           accept_len, next_token, margins);
        BS_LAUNCH_CHECK();
        return BS_OK;
    }
    float2* stats = reinterpret_cast<float2*>(stats_scratch);
    const float inv_temp = 1.0f / temperature;
    if (dtype == BS_BF16)
        hipLaunchKernelGGL((row_stats_kernel<uint16_t>), dim3(n_rows), dim3(256), 0, stream, (const uint16_t*)p_logits,
                           (const uint16_t*)q_logits, n_p, V, inv_temp, stats);
    else
        hipLaunchKernelGGL((row_stats_kernel<float>), dim3(n_rows), dim3(256), 0, stream, (const float*)p_logits,
                           (const float*)q_logits, n_p, V, inv_temp, stats);
    BS_LAUNCH_CHECK();
    DecideParams a;
    a.p_logits = p_logits; a.q_logits = q_logits; a.draft_tokens = draft_tokens; a.uniforms = uniforms; a.seed = seed;
    a.round_ptr = round_ptr; a.round = round; a.gamma = gamma; a.V = V; a.n_p_rows = n_p; a.inv_temp = inv_temp;
    a.stats = stats; a.flags = flags; a.cand = cand; a.accept_len = accept_len; a.next_token = next_token; a.margins = margins;
    // The deciding row pair is streamed again (it was read a moment ago by phase A: L2 / memory-side cache), not kept
    // in registers: 42 instead of 256 registers per lane lets several sequences share a compute unit, which is what
    // hides this kernel's chain of dependent loads (measured at B = 1024: 77 -> 42 us).
    const dim3 grid(B), block(ST);
    if (dtype == BS_BF16) hipLaunchKernelGGL((spec_decide_kernel<uint16_t, 1, false>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((spec_decide_kernel<float, 1, false>), grid, block, 0, stream, a);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

}  // namespace bs

extern "C" __attribute__((visibility("default"))) size_t bs_spec_sample_workspace_bytes(int B, int gamma) {
    if (B < 0 || gamma < 0) return 0;
    return bs::spec_scratch_bytes(B, gamma);
}

// Argument checks shared by the two entry points (everything but the scratch memory).
static int check_spec_sample_args(const char* who, const void* dev_target_logits, const void* dev_draft_logits,
                                  const int32_t* dev_draft_tokens, int B, int gamma, int V, int dtype, float temperature,
                                  const int32_t* dev_accept_len, const int32_t* dev_next_token) {
    BS_REQUIRE(B >= 0 && gamma >= 0, BS_EINVAL, "%s: B=%d gamma=%d must be >= 0", who, B, gamma);
    BS_REQUIRE(V >= 1 && V <= (1 << 20), BS_ESHAPE, "%s: V=%d outside [1, 2^20]", who, V);
    BS_REQUIRE(gamma <= 512, BS_ESHAPE, "%s: gamma=%d > 512", who, gamma);
    BS_REQUIRE((long long)B * (gamma + 1) < (1LL << 31), BS_ESHAPE, "%s: B*(gamma+1) overflows", who);
    BS_REQUIRE(dtype == BS_F32 || dtype == BS_BF16, BS_EDTYPE, "%s: dtype %d", who, dtype);
    BS_REQUIRE(temperature >= 0.f && isfinite(temperature), BS_EINVAL, "%s: temperature %g", who, (double)temperature);
    if (B == 0) return BS_OK;
    BS_REQUIRE(dev_target_logits && dev_accept_len && dev_next_token, BS_EINVAL, "%s: NULL pointer", who);
    BS_REQUIRE(gamma == 0 || (dev_draft_tokens && (dev_draft_logits || temperature == 0.f)), BS_EINVAL, "%s: NULL draft input", who);
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_spec_sample(const void* dev_target_logits, const void* dev_draft_logits,
                              const int32_t* dev_draft_tokens, int B, int gamma, int V, int dtype, float temperature,
                              const float* dev_uniforms, uint64_t seed, uint32_t round, int32_t* dev_accept_len,
                              int32_t* dev_next_token, float* dev_margins, void* dev_workspace,
                              size_t workspace_bytes, void* stream) {
    const int rc = check_spec_sample_args("bs_spec_sample", dev_target_logits, dev_draft_logits, dev_draft_tokens, B, gamma, V, dtype,
                                          temperature, dev_accept_len, dev_next_token);
    if (rc != BS_OK || B == 0) return rc;
    BS_REQUIRE(dev_workspace, BS_EINVAL, "bs_spec_sample: NULL pointer");
    BS_REQUIRE(workspace_bytes >= bs_spec_sample_workspace_bytes(B, gamma), BS_EWORKSPACE,
               "bs_spec_sample: workspace %zu < %zu bytes", workspace_bytes, bs_spec_sample_workspace_bytes(B, gamma));
    BS_REQUIRE((reinterpret_cast<uintptr_t>(dev_workspace) & 15) == 0, BS_EWORKSPACE, "bs_spec_sample: workspace misaligned");
    return bs::launch_spec_sample(dev_target_logits, dev_draft_logits, dev_draft_tokens, B, gamma, V, dtype, temperature,
                                  dev_uniforms, seed, nullptr, round, dev_workspace, nullptr, nullptr, dev_accept_len,
                                  dev_next_token, dev_margins, reinterpret_cast<hipStream_t>(stream));
}

// ---- the same call for callers that cannot allocate: the per-row statistics live in a static device array ----------
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process ends.  The
// array's name is only a host-side handle: the address the kernels get is looked up once per device.
namespace {
constexpr int STATIC_ROWS = 65536;                         // logit rows B * (2 gamma + 1) one call may have: 512 KiB
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) float2 scratch[STATIC_ROWS];
void* g_scratch_ptr[STATIC_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

int static_scratch(void** out) {
    int dev = -1;
    BS_HIP(hipGetDevice(&dev));
    BS_REQUIRE(dev >= 0 && dev < STATIC_MAX_DEVICES, BS_ESTATE, "bs_spec_sample_static: device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        BS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // this device's copy (the current device)
        BS_REQUIRE(p, BS_EHIP, "bs_spec_sample_static: no address for the static scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return BS_OK;
}
}  // namespace

extern "C" __attribute__((visibility("default"))) size_t bs_spec_sample_static_max_rows(void) { return STATIC_ROWS; }

extern "C" __attribute__((visibility("default"))) int bs_spec_sample_static(const void* dev_target_logits, const void* dev_draft_logits,
                              const int32_t* dev_draft_tokens, int B, int gamma, int V, int dtype, float temperature,
                              const float* dev_uniforms, uint64_t seed, uint32_t round, int32_t* dev_accept_len,
                              int32_t* dev_next_token, float* dev_margins, void* stream) {
    int rc = check_spec_sample_args("bs_spec_sample_static", dev_target_logits, dev_draft_logits, dev_draft_tokens, B, gamma, V, dtype,
                                    temperature, dev_accept_len, dev_next_token);
    if (rc != BS_OK || B == 0) return rc;
    BS_REQUIRE((long long)B * (2 * gamma + 1) <= STATIC_ROWS, BS_ESHAPE,
               "bs_spec_sample_static: B*(2*gamma+1) = %lld logit rows exceed the static scratch of %d rows; use bs_spec_sample",
               (long long)B * (2 * gamma + 1), STATIC_ROWS);
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != BS_OK) return rc;
    // nothing in the scratch has to start at zero: phase A writes every row's statistics before phase B reads them
    return bs::launch_spec_sample(dev_target_logits, dev_draft_logits, dev_draft_tokens, B, gamma, V, dtype, temperature,
                                  dev_uniforms, seed, nullptr, round, ws, nullptr, nullptr, dev_accept_len,
                                  dev_next_token, dev_margins, reinterpret_cast<hipStream_t>(stream));
}
