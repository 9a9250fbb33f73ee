// One launch = one forward pass of a small model over one or two rows (a draft step of App. A: x~_i ~ Q(. | pt, x~_{<i});
// also a step of canonical decoding, Alg. 1, when the model is small enough).
//
// With a handful of rows every kernel of a layer is a few microseconds of latency and nothing else.  Measured on the
// 12-layer 768-wide draft: a kernel boundary costs 1.6 us, the first load of a fresh kernel 2.2 us (kernel arguments,
// cold translation, data another die wrote), the last store's acknowledgement 0.8-1.9 us, and the weights cannot be
// requested before the kernel starts: 5.5-7 us per kernel, 61 kernels per step.  A grid barrier between phases of one
// resident kernel does not help by itself (acknowledged stores 1.9 us + arrival counter and poll 1 us + reload 1.1 us).
// Here ONE resident kernel walks all phases of all layers
//
//   QKV projection -> attention (split over keys) -> O projection + residual -> gate/up + SwiGLU -> down + residual
//
// WITHOUT barriers: what one phase hands to the next lives in small exchange buffers of 8-byte cells {value, flag},
// written and read with device-scope (sc1) accesses (the L2 of a die is not coherent with the others).  A consumer
// polls the cells it needs until they carry the flag of the producing phase, so the hand-over costs one store and one
// load, nobody waits for acknowledgements, and a workgroup that has no part in a phase walks past it.  The flags are
// cleared by the prep kernel ahead of every launch.  Re-use of a buffer needs no barrier either: between two writes of
// the same buffer lies at least one phase whose every workgroup consumed ALL of the previous phase's output, so every
// reader of the old contents has finished before the first writer of the new ones can start (spelled out at the phase
// loop).  A workgroup requests the weights of its next phase (and the cached keys and values of its attention unit)
// before it starts polling, so they travel while it waits.
// Every projection phase is the few-row projection of gemm_dec_kernel: a workgroup owns 16 output columns over the
// whole K, its 8 wavefronts split K and add through LDS, wavefront 0 finishes the columns.  RMSNorm needs no partial
// sums here: every workgroup stages the whole input rows (gain . x, as soon as x is there) and adds up their squares
// itself; the row's scale is applied in the epilogue.
// At this size the instruction stream counts as much as the memory system: one wavefront retires a dependent
// instruction every 4-8 cycles, so a few hundred instructions between "the input is there" and "the output is stored"
// are a microsecond per phase.  What the phase loop needs is therefore worked out ahead of the polls, loops with
// run-time bounds are kept off that path, and there is one tile per workgroup and phase.
#include <math.h>
#include "common.h"
#include "kernels.h"
#include "devutil.h"

namespace bs {

constexpr int STEP_WAVES = 8, STEP_THREADS = 64 * STEP_WAVES;
constexpr int STEP_MAXS = 16;            // k steps of 32 columns one wavefront may own in a phase (K <= 4096)
constexpr int STEP_XR = 4;               // groups of four staged input values per lane (2 rows x 4096 columns / 4 / 512 lanes)
constexpr int STEP_MB = 5;               // attention partials the O projection's staging merges per round of polls
constexpr int STEP_XCOPIES = 2;          // copies of the residual stream's exchange cells: every workgroup of a phase polls all of them
constexpr int STEP_BLK = 1;              // key blocks a wavefront of an attention unit takes before more splits are used

// tiled weights: byte offset of lane (row local % 16, k-slot lq) in the 16-row tile that holds row `local`; a k step is
// 4096 bytes further.  Every matrix is below 4 GiB (host check), so the offset is 32-bit and the matrix base stays scalar.
__device__ __forceinline__ uint32_t step_tile_off(int local, int K, int lq) {
    return (uint32_t)(((size_t)(local >> 6) * 64 * K + ((local >> 4) & 3) * 512 + ((local & 15) + 16 * lq) * 8) * 2);
}

enum { PH_QKV = 0, PH_ATT = 1, PH_O = 2, PH_GU = 3, PH_DOWN = 4, PH_PER_LAYER = 5 };
__device__ __forceinline__ unsigned step_flag(int l, int kind) { return 1u + (unsigned)(l * PH_PER_LAYER + kind); }

template <int HD>
__global__ __launch_bounds__(STEP_THREADS) void dec_step_kernel(StepArgs a) {
    constexpr int DS = HD / 32, DT = HD / 16;
    constexpr int PCELLS = HD + 4;                                      // cells of one attention partial: o[HD], max, sum, 2 pad
    __shared__ __attribute__((aligned(16))) float red[STEP_WAVES][256];
    __shared__ float s_part[STEP_WAVES][2];
    __shared__ int s_abort;
    extern __shared__ __attribute__((aligned(16))) uint16_t xs[];       // [2 planes][M][Kp]; the attention phase reuses it
    // Code size matters here: the instruction cache holds 64 KB for two compute units and every layer walks the whole
    // phase loop, so every helper below has one or two call sites and the row / query arithmetic uses that there are at
    // most two rows (no integer divisions).
    // The lane indices are passed through an empty asm at the top of every phase: without that the compiler hoists the
    // index arithmetic of all phases out of the phase loop and spills hundreds of registers around it.
    int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform: branches on it are scalar
    const int G = gridDim.x, wg = blockIdx.x;
    const int M = a.M, d = a.d, ff = a.ff, H = a.H, KVH = a.KVH, q_len = a.q_len;
    const int qs = q_len - 1;                                           // q_len is 1 or 2: r / q_len = r >> qs, r % q_len = r & qs
    const int nq = H * HD, nkv = KVH * HD, nqkv = nq + 2 * nkv;
    const int Gq = H / KVH, R = Gq * q_len;
    const int Kp = a.kp;                                                // padded plane row, elements
    const unsigned limit = a.spin_limit;
    bool row_ok = li < M;
    if (tid == 0) s_abort = 0;
    __syncthreads();
    // The residual stream is polled by every workgroup of the QKV, gate/up and logits phases: its cells exist in
    // STEP_XCOPIES copies (the producers store each), and a workgroup reads the copy of its parity -- half the readers per
    // memory channel (measured with an all-to-all of such cells: 2.06 -> 1.86 us for 12 KB among 256 workgroups).
    const int xcopy = (wg % STEP_XCOPIES) * (M * d);
    const DevBuf bX = dev_buf(a.X), bQ = dev_buf(a.Q), bKVN = dev_buf(a.KVN), bPA = dev_buf(a.PA), bACT = dev_buf(a.ACT);

    // A poll that ran out of patience (a producer that never came: only if the workgroups are not all resident, or after a
    // fault elsewhere): remember it, finish the phase with whatever was read, leave at the next workgroup-wide check.
    auto alive = [&]() -> bool {                        // workgroup-wide: call where all wavefronts pass
        __syncthreads();
        if (s_abort == 0) return true;
        if (tid == 0) atomicOr(a.status, 16);
        return false;
    };
    // four consecutive cells, polled until all carry `flag`
    auto poll4 = [&](DevBuf b, int c, unsigned flag) -> float4 {
        u32x4 lo, hi;
        unsigned spins = 0;
        while (true) {
            asm volatile("" ::: "memory");              // the cells change under our feet: every round reads memory again
            lo = ld_cells2(b, c); hi = ld_cells2(b, c + 2);
            if (lo.y == flag && lo.w == flag && hi.y == flag && hi.w == flag) break;
            if (++spins > limit) { s_abort = 1; break; }
        }
        return make_float4(__uint_as_float(lo.x), __uint_as_float(lo.z), __uint_as_float(hi.x), __uint_as_float(hi.z));
    };

    // N groups of four cells: all loads of a round are in flight together (a round trip takes half a microsecond when the
    // data is there; polls one after the other would add up).  Cell index < 0: not wanted, zeros.
    auto poll4n = [&](DevBuf b, auto& cells, unsigned flag, auto& out) {
        constexpr int N = sizeof(cells) / sizeof(cells[0]);
        u32x4 lo[N], hi[N];
        unsigned spins = 0;
        while (true) {
            asm volatile("" ::: "memory");
            bool ok = true;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                // nothing is loaded for an entry that is not wanted: a dummy address would be the same for every lane of
                // every workgroup, and such a hot spot costs microseconds
                if (cells[i] >= 0) { lo[i] = ld_cells2(b, cells[i]); hi[i] = ld_cells2(b, cells[i] + 2); }
                else { lo[i] = u32x4{0u, flag, 0u, flag}; hi[i] = lo[i]; }
                ok = ok && (lo[i].y == flag && lo[i].w == flag && hi[i].y == flag && hi[i].w == flag);
            }
            if (ok) break;
            if (++spins > limit) { s_abort = 1; break; }
        }
#pragma unroll
        for (int i = 0; i < N; ++i)
            out[i] = cells[i] < 0 ? make_float4(0.f, 0.f, 0.f, 0.f)
                                  : make_float4(__uint_as_float(lo[i].x), __uint_as_float(lo[i].z), __uint_as_float(hi[i].x), __uint_as_float(hi[i].z));
    };

    // ---- a wavefront's share of a projection: K steps [s0, s0 + n) of a 16-row weight tile -------------------------
    // Requested in groups of four steps behind one scalar branch each; every entry is defined on every path (a group
    // past the share is zero, a step past it repeats the last one and is multiplied as zero), so that nothing of an
    // earlier phase stays live in these registers.
    uint4 wp[STEP_MAXS];
    auto wfetch = [&](const uint16_t* w, uint32_t lane_off, int s0, int n) {
        const char* wb = reinterpret_cast<const char*>(w);
        const uint32_t off = lane_off + (uint32_t)s0 * 4096u;
#pragma unroll
        for (int g = 0; g < STEP_MAXS / 4; ++g) {
            if (4 * g < n) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    wp[4 * g + j] = ldg16(reinterpret_cast<const uint16_t*>(wb + (off + (uint32_t)min(4 * g + j, n - 1) * 4096u)));
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) wp[4 * g + j] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    // the lane's B operand of k step s0 (hi plane; the lo plane is M * Kp elements further), as an element offset into xs
    auto plane_off = [&](int s0) -> int { return min(li, M - 1) * Kp + lq * 8 + s0 * 32; };
    auto wmma = [&](int boff, int n) -> f32x4 {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};             // hi and lo plane: two independent chains
        const uint16_t* bh = xs + boff;
        const uint16_t* bl = bh + (size_t)M * Kp;
#pragma unroll
        for (int g = 0; g < STEP_MAXS / 4; ++g) {
            if (4 * g < n) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int u = 4 * g + j, ub = min(u, n - 1);
                    uint4 wv = wp[u];
                    if (u >= n) wv = make_uint4(0u, 0u, 0u, 0u);
                    const bf16x8 A = __builtin_bit_cast(bf16x8, wv);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bh + ub * 32)), acc, 0, 0, 0);
                    acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(bl + ub * 32)), acl, 0, 0, 0);
                }
            }
        }
        acc[0] += acl[0]; acc[1] += acl[1]; acc[2] += acl[2]; acc[3] += acl[3];
        return acc;
    };
    // planes (hi, lo) of four consecutive values of row m at column c
    auto put_planes = [&](int m, int c, float v0, float v1, float v2, float v3) {
        const uint16_t h0 = from_f<uint16_t>(v0), h1 = from_f<uint16_t>(v1), h2 = from_f<uint16_t>(v2), h3 = from_f<uint16_t>(v3);
        *reinterpret_cast<uint2*>(&xs[(size_t)m * Kp + c]) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
        *reinterpret_cast<uint2*>(&xs[(size_t)(M + m) * Kp + c]) =
            make_uint2(pack_bf16(v0 - to_f(h0), v1 - to_f(h1)), pack_bf16(v2 - to_f(h2), v3 - to_f(h3)));
    };

    // r of row m from the wavefronts' partial sums of squares (valid behind the staging barrier of a normed phase)
    const float inv_d = 1.0f / (float)d;
    auto row_scale = [&](int m) -> float {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < STEP_WAVES; ++w) t += s_part[w][m];
        return __builtin_amdgcn_rsqf(t * inv_d + a.eps);     // one instruction, 1 ulp: this sits in the epilogue, on the critical path
    };

    // ---- per-row facts from the prep kernel (positions, tokens) ----------------------------------------------------------
    const int m_row = min(li, M - 1);
    const int p_row = a.pos[m_row];
    const int b_row = m_row >> qs;
    const int tok_row = a.tok[m_row];

    // ---- attention unit of this workgroup (the same in every layer) --------------------------------------------------------
    // Units: per (sequence, kv head) one for the keys of this pass's own rows (they arrive through the exchange cells) and S
    // for splits of the cached keys, of which only as many are used as leave a wavefront STEP_BLK blocks of 32 keys;
    // producer (attention) and consumer (O projection) derive that number from the sequence's cache length alike.  The
    // units sit behind the QKV tiles, own-key units first, then split 0 of all heads, split 1, ..: the used ones are the
    // lowest, and a workgroup rarely has a part in two consecutive phases.
    const int S = a.splits;
    const int n_bk = a.B * KVH;
    const int att_unit = (wg - (nqkv / 16) % G + G) % G;
    int at_b = 0, at_kvh = 0, at_s = 0, at_pos0 = -1, blk0 = 0, blk_end = 0;
    auto used_splits = [&](int pos0) -> int {
        const int nblk = pos0 > 0 ? (pos0 + 31) >> 5 : 0;
        const int want = (nblk + STEP_WAVES * STEP_BLK - 1) / (STEP_WAVES * STEP_BLK);
        return max(1, min(S, want));
    };
    bool att_active = false, att_own = false;
    if (att_unit < n_bk * (S + 1)) {
        const int bk = att_unit % n_bk;
        at_b = bk / KVH;
        at_kvh = bk - at_b * KVH;
        at_s = att_unit / n_bk - 1;                         // -1: the own keys
        at_pos0 = a.pos[at_b * q_len];                      // keys already in the cache; -1: sequence left out
        att_own = at_s < 0;
        if (att_own) {
            at_s = S;                                       // its partial sits behind the splits
            att_active = true;
        } else {
            const int nblk = at_pos0 > 0 ? (at_pos0 + 31) >> 5 : 0;
            const int Se = used_splits(at_pos0);
            const int per = (nblk + Se - 1) / Se;
            blk0 = at_s * per + wave;
            blk_end = at_s < Se ? min(nblk, (at_s + 1) * per) : 0;
            att_active = at_s < Se;
        }
    }
    const int Se_row0 = used_splits(a.pos[0]), Se_row1 = used_splits(a.pos[(M - 1) >> qs << qs]);     // splits of row 0's / row 1's sequence

    const int nt_qkv = nqkv / 16, nt_o = d / 16, nt_gu = ff / 16;
    const int n_ph = a.n_layers * PH_PER_LAYER;             // phase n_ph = the logits
    const bool lm_on = a.logit_rows > 0;
    auto tiles_of = [&](int kind) -> int { return kind == PH_QKV ? nt_qkv : (kind == PH_GU ? nt_gu : (kind == PH_ATT ? 0 : nt_o)); };
    // first tile of this workgroup in a projection phase: QKV and gate/up tiles are dealt from workgroup 0 upwards, O and
    // down tiles from the last workgroup downwards, the attention units sit behind the QKV tiles: a workgroup rarely has
    // work in two consecutive phases, so the weights of its next tile are on their way a whole phase early
    auto first_tile = [&](int kind) -> int { return (kind == PH_O || kind == PH_DOWN) ? G - 1 - wg : wg; };
    // weights of tile u of phase (l, kind) for this wavefront
    auto fetch_tile = [&](int l, int kind, int u) {
        const int K = kind == PH_O ? nq : (kind == PH_DOWN ? ff : d), steps = K >> 5;
        const uint16_t* w;
        int local0 = u * 16, wv = wave, wsh = 3;            // 8 wavefronts share K (gate / up: 4 each)
        if (kind == PH_QKV) {
            if (local0 < nq) w = a.w[l][0];
            else if (local0 < nq + nkv) { w = a.w[l][1]; local0 -= nq; }
            else { w = a.w[l][2]; local0 -= nq + nkv; }
        } else if (kind == PH_O) w = a.w[l][3];
        else if (kind == PH_GU) { wsh = 2; w = a.w[l][4 + (wave >> 2)]; wv = wave & 3; }
        else w = a.w[l][6];
        const int s0 = (wv * steps) >> wsh, n = (((wv + 1) * steps) >> wsh) - s0;
        wfetch(w, step_tile_off(local0 + li, K, lq), s0, n);
    };
    int want_ph = 0, want_u = -1;                           // the next projection tile of this workgroup: phase and tile
    int have_ph = -1, have_u = -1;                          // what sits in wp
    // next projection phase >= p in which this workgroup owns a tile (a layer ahead at most)
    auto next_own = [&](int p) {
        want_ph = 1 << 30; want_u = -1;
        for (int p2 = p; p2 < p + PH_PER_LAYER + 1 && p2 < n_ph; ++p2) {
            const int k2 = p2 % PH_PER_LAYER;
            if (k2 != PH_ATT && first_tile(k2) < tiles_of(k2)) { want_ph = p2; want_u = first_tile(k2); return; }
        }
    };
    next_own(0);

    // ============================== the phases ================================================================================
    // Buffer re-use without barriers (F(l,k) = flag of phase k of layer l):
    //   X    written by O(l) [F(l,O)] and DOWN(l) [F(l,DOWN)], each cell by the workgroup that owns its column.  Readers of
    //        the value before O(l) writes: QKV(l) workgroups; O(l) needs all attention partials, which need all of Q, which
    //        every QKV(l) workgroup wrote after it had read X.  Readers before DOWN(l) writes: GU(l) workgroups; DOWN(l)
    //        needs all of ACT, written by them after reading X.
    //   Q, KVN written by QKV(l+1): their readers, the attention units of layer l, all finished before any O(l) tile could,
    //        and QKV(l+1) is three all-to-all phases later.  PA (ATT -> O) and ACT (GU -> DOWN) likewise.
    for (int ph = 0; ph <= n_ph; ++ph) {
        asm volatile("" : "+v"(tid));
        lane = tid & 63; li = lane & 15; lq = lane >> 4;
        row_ok = li < M;
        // the weights of this workgroup's next tile are requested as early as the registers are free: here, at the top of
        // every phase (one call site), i.e. right after the previous tile's multiply
        if (want_ph < ph) next_own(ph);
        if (want_u >= 0 && (have_ph != want_ph || have_u != want_u)) {
            fetch_tile(want_ph / PH_PER_LAYER, want_ph % PH_PER_LAYER, want_u);
            have_ph = want_ph; have_u = want_u;
        }
        const int l = ph / PH_PER_LAYER, kind = ph - l * PH_PER_LAYER;
        const bool is_lm = ph == n_ph;
        if (is_lm && !lm_on) break;
        char* kc = a.kv + (size_t)l * a.kv_layer;
        char* vc = kc + a.kv_layer / 2;
        if (!is_lm && kind == PH_ATT) {
            // ================= attention of the new rows against the cache, one split of the keys per unit =================
            if (!att_active) continue;
            float* wm = reinterpret_cast<float*>(xs);                           // [waves][16]
            float* wl = wm + STEP_WAVES * 16;                                   // [waves][16]
            float* wo = wl + STEP_WAVES * 16;                                   // [waves][R][HD + 1]
            uint4* sq = reinterpret_cast<uint4*>(wo + STEP_WAVES * R * (HD + 1));  // [2 planes][DS][64 lanes]: the queries as MFMA operands
            const int m_first = at_b * q_len;
            const unsigned fin = step_flag(l, PH_QKV), fout = step_flag(l, PH_ATT);
            const char* kbb = kc + (((size_t)at_b * KVH + at_kvh) * (size_t)a.cache_len * HD) * 2;
            const char* vbb = vc + (((size_t)at_b * KVH + at_kvh) * (size_t)a.cache_len * HD) * 2;
            const bool rvalid = li < R && at_pos0 >= 0;
            const int g_r = rvalid ? li >> qs : 0, qi_r = rvalid ? li & qs : 0;
            float m_run = -INFINITY, l_run = 0.f;
            f32x4 o[DT];
#pragma unroll
            for (int t = 0; t < DT; ++t) o[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            {
                // this wavefront's blocks: its share of the split's cached keys (the first requested up front, before
                // anything is polled for), or (own-key unit, wavefront 0) the keys of this pass's own rows as one block;
                // none for a sequence that was left out (at_pos0 < 0: no cached blocks either), which still waits below
                const int n_old = (!att_own && blk0 < blk_end) ? (blk_end - blk0 + STEP_WAVES - 1) / STEP_WAVES : 0;
                const int n_it = at_pos0 < 0 ? 0 : (att_own ? (wave == 0 ? 1 : 0) : n_old);
                uint4 kfa[STEP_BLK][2][DS], vfa[STEP_BLK][DT], qh[DS], ql[DS];
                auto old_fetch = [&](int blk, uint4 (&kf)[2][DS], uint4 (&vf)[DT]) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int krow = min(blk * 32 + t * 16 + li, at_pos0 - 1);
#pragma unroll
                        for (int ds = 0; ds < DS; ++ds)
                            kf[t][ds] = ldg16(reinterpret_cast<const uint16_t*>(kbb + (uint32_t)((krow * HD + ds * 32 + lq * 8) * 2)));
                    }
#pragma unroll
                    for (int t = 0; t < DT; ++t)
                        vf[t] = ldg16(reinterpret_cast<const uint16_t*>(vbb + (uint32_t)((((blk * HD + t * 16 + li) * 32) + lq * 8) * 2)));
                };
#pragma unroll
                for (int j = 0; j < STEP_BLK; ++j) {
                    if (j < n_old) old_fetch(blk0 + j * STEP_WAVES, kfa[j], vfa[j]);
                    else {
#pragma unroll
                        for (int t = 0; t < 2; ++t)
#pragma unroll
                            for (int ds = 0; ds < DS; ++ds) kfa[j][t][ds] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                        for (int t = 0; t < DT; ++t) vfa[j][t] = make_uint4(0u, 0u, 0u, 0u);
                    }
                }
                // The queries of this unit's rows and, for an own-key unit, the keys and values of this pass's rows (they arrive
                // together, from the QKV phase): one round of loads, addressed relative to the query buffer.
                // Key j = li of this pass (row m_first + j).  Values: lane (dimension 16t + li, k-slot lq) holds keys
                // (e >> 2) * 16 + 4 lq + (e & 3), so only k-slot 0, e < q_len exist; lane (li, lq) polls for the tiles
                // t = lq, lq + 4, .. (four cells of dimensions 4 * (li / 4) .., the lane keeps its own) and k-slot 0 collects them.
                // Wavefront 0 polls for the whole unit and hands the queries on through LDS: eight wavefronts polling each for
                // itself see the data up to a round trip apart, and the unit is as late as its last one.
                constexpr int NQ = 2 * DS, NK = 2 * DS, NV = DT / 2;
                float4 kv_[NK + NV];
                if (wave == 0) {
                    const float scale = 1.0f / sqrtf((float)HD);
                    const int kvn_rel = (int)((reinterpret_cast<const char*>(a.KVN) - reinterpret_cast<const char*>(a.Q)) >> 3);
                    int qc[NQ + NK + NV];
                    float4 qo[NQ + NK + NV];
#pragma unroll
                    // It polls whether or not anybody has a block to multiply the queries with, also for a sequence that was
                    // left out (the QKV phase writes query cells for every row): a unit must not write its partial before the
                    // QKV phase of this layer has run, or it would overwrite what the O projection of the layer before is still
                    // reading (a unit without any cached key would run layers ahead).
                    for (int i = 0; i < NQ; ++i) qc[i] = ((m_first + qi_r) * H + at_kvh * Gq + g_r) * HD + (i >> 1) * 32 + lq * 8 + (i & 1) * 4;
#pragma unroll
                    for (int i = 0; i < NK; ++i)
                        qc[NQ + i] = (att_own && n_it > 0 && li < q_len)
                                         ? kvn_rel + (m_first + li) * 2 * nkv + at_kvh * HD + (i >> 1) * 32 + lq * 8 + (i & 1) * 4 : -1;
#pragma unroll
                    for (int i = 0; i < NV; ++i)
                        qc[NQ + NK + i] = (att_own && n_it > 0 && ((i & 1) == 0 || q_len > 1))
                                              ? kvn_rel + (m_first + (i & 1)) * 2 * nkv + nkv + at_kvh * HD + (lq + 4 * (i >> 1)) * 16 + (li & ~3) : -1;
                    poll4n(bQ, qc, fin, qo);
                    float4 qv[NQ];
#pragma unroll
                    for (int i = 0; i < NQ; ++i) qv[i] = qo[i];
#pragma unroll
                    for (int i = 0; i < NK + NV; ++i) kv_[i] = qo[NQ + i];
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) {
                        float v[8] = {qv[2 * ds].x, qv[2 * ds].y, qv[2 * ds].z, qv[2 * ds].w, qv[2 * ds + 1].x, qv[2 * ds + 1].y, qv[2 * ds + 1].z, qv[2 * ds + 1].w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = rvalid ? v[e] * scale : 0.f;
                        split8(v, qh[ds], ql[ds]);
                        sq[ds * 64 + lane] = qh[ds];
                        sq[(DS + ds) * 64 + lane] = ql[ds];
                    }
                }
                if (!alive()) return;
                if (wave != 0) {
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) { qh[ds] = sq[ds * 64 + lane]; ql[ds] = sq[(DS + ds) * 64 + lane]; }
                }
                for (int it = 0; it < n_it; ++it) {
                    const bool own = it >= n_old;
                    uint4 kf[2][DS], vf[DT];
                    int n_vis;
                    if (!own) {
                        const int blk = blk0 + it * STEP_WAVES;
                        n_vis = min(32, at_pos0 - blk * 32);
                        if (it < STEP_BLK) {                                    // requested up front (static register selection)
#pragma unroll
                            for (int j = 0; j < STEP_BLK; ++j)
                                if (j == it) {
#pragma unroll
                                    for (int t = 0; t < 2; ++t)
#pragma unroll
                                        for (int ds = 0; ds < DS; ++ds) kf[t][ds] = kfa[j][t][ds];
#pragma unroll
                                    for (int t = 0; t < DT; ++t) vf[t] = vfa[j][t];
                                }
                        } else {
                            old_fetch(blk, kf, vf);                             // more blocks than were foreseen: one at a time
                        }
                    } else {
                        n_vis = q_len;                                           // the keys are bf16 already: the hi plane is exact
#pragma unroll
                        for (int ds = 0; ds < DS; ++ds) {
                            const float4 k0 = kv_[2 * ds], k1 = kv_[2 * ds + 1];
                            kf[0][ds] = make_uint4(pack_bf16(k0.x, k0.y), pack_bf16(k0.z, k0.w), pack_bf16(k1.x, k1.y), pack_bf16(k1.z, k1.w));
                            kf[1][ds] = make_uint4(0u, 0u, 0u, 0u);
                        }
                        const int sub = li & 3;
                        uint32_t packed[DT / 4];
#pragma unroll
                        for (int i = 0; i < DT / 4; ++i) {
                            const float4 q4 = kv_[NK + 2 * i], r4 = kv_[NK + 2 * i + 1];
                            const float v0 = sub == 0 ? q4.x : (sub == 1 ? q4.y : (sub == 2 ? q4.z : q4.w));
                            const float v1 = sub == 0 ? r4.x : (sub == 1 ? r4.y : (sub == 2 ? r4.z : r4.w));
                            packed[i] = pack_bf16(v0, v1);
                        }
#pragma unroll
                        for (int t = 0; t < DT; ++t)                              // slots of k-slots 1..3 are zeroed below (n_vis <= 2)
                            vf[t] = make_uint4((uint32_t)__shfl((int)packed[t >> 2], li + 16 * (t & 3), 64), 0u, 0u, 0u);
                    }
                    // ---- one block of 32 keys: scores, online softmax, values.  n_vis keys exist; own keys are causal ----
                    if (n_vis < 32) {                                           // slots past the end may hold anything: zero them
#pragma unroll
                        for (int t = 0; t < DT; ++t) {
                            uint32_t w[4] = {vf[t].x, vf[t].y, vf[t].z, vf[t].w};
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const int key = (e >> 2) * 16 + 4 * lq + (e & 3);
                                if (key >= n_vis) w[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                            }
                            vf[t] = make_uint4(w[0], w[1], w[2], w[3]);
                        }
                    }
                    f32x4 sc[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        sc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ds = 0; ds < DS; ++ds) {
                            const bf16x8 A = __builtin_bit_cast(bf16x8, kf[t][ds]);
                            sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, qh[ds]), sc[t], 0, 0, 0);
                            sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, ql[ds]), sc[t], 0, 0, 0);
                        }
                    }
                    float sv[8], bm = -INFINITY;
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int key = t * 16 + 4 * lq + e;
                            const bool vis = rvalid && key < n_vis && (!own || key <= qi_r);
                            sv[t * 4 + e] = vis ? sc[t][e] : -INFINITY;
                            bm = fmaxf(bm, sv[t * 4 + e]);
                        }
                    bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
                    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
                    const float m_new = fmaxf(m_run, bm);
                    float pv[8], alpha = 1.f, psum = 0.f;
                    if (m_new == -INFINITY) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) pv[e] = 0.f;
                    } else {
                        alpha = __expf(m_run - m_new);
#pragma unroll
                        for (int e = 0; e < 8; ++e) { pv[e] = __expf(sv[e] - m_new); psum += pv[e]; }
                    }
                    l_run = l_run * alpha + psum;
                    m_run = m_new;
                    uint4 ph_, pl_;
                    split8(pv, ph_, pl_);
#pragma unroll
                    for (int t = 0; t < DT; ++t) {
                        o[t][0] *= alpha; o[t][1] *= alpha; o[t][2] *= alpha; o[t][3] *= alpha;
                        const bf16x8 A = __builtin_bit_cast(bf16x8, vf[t]);
                        o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, ph_), o[t], 0, 0, 0);
                        o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8, pl_), o[t], 0, 0, 0);
                    }
                }
            }
            // ---- combine the wavefronts: lane holds O^T[d = 16t + 4lq + e][row li]; a sequence that was left out, or a
            //      wavefront without blocks, contributes (max = -inf, sum = 0, o = 0) ----
            float lr = l_run;
            lr += __shfl_xor(lr, 16, 64);
            lr += __shfl_xor(lr, 32, 64);
            if (lq == 0) { wm[wave * 16 + li] = m_run; wl[wave * 16 + li] = lr; }
            if (li < R) {
#pragma unroll
                for (int t = 0; t < DT; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) wo[((size_t)wave * R + li) * (HD + 1) + t * 16 + 4 * lq + e] = o[t][e];
            }
            if (!alive()) return;
            // eight consecutive lanes = the eight wavefronts' shares of two output dimensions of one row: each reads its
            // wavefront's (max, sum, two outputs), three shuffles find the maximum, three add the rescaled shares, and the
            // first of the eight stores two cells with one 16-byte store
            for (int base = 0; base < R * (HD / 2); base += STEP_THREADS / STEP_WAVES) {
                const int idx = base + (tid >> 3), w = tid & 7;
                const bool on = idx < R * (HD / 2);
                const int r = on ? idx / (HD / 2) : 0, dd = on ? (idx % (HD / 2)) * 2 : 0;
                const float mw = wm[w * 16 + r];
                float mm = mw;
                mm = fmaxf(mm, __shfl_xor(mm, 1, 64)); mm = fmaxf(mm, __shfl_xor(mm, 2, 64)); mm = fmaxf(mm, __shfl_xor(mm, 4, 64));
                const float f = (mw == -INFINITY) ? 0.f : __expf(mw - mm);
                float ov0 = wo[((size_t)w * R + r) * (HD + 1) + dd] * f, ov1 = wo[((size_t)w * R + r) * (HD + 1) + dd + 1] * f;
                float lv = wl[w * 16 + r] * f;
#pragma unroll
                for (int o_ = 1; o_ < 8; o_ <<= 1) {
                    ov0 += __shfl_xor(ov0, o_, 64); ov1 += __shfl_xor(ov1, o_, 64); lv += __shfl_xor(lv, o_, 64);
                }
                if (on && w == 0) {
                    const int c = (((m_first + (r & qs)) * H + at_kvh * Gq + (r >> qs)) * (S + 1) + at_s) * PCELLS;
                    st_cells2(bPA, c + dd, ov0, ov1, fout);
                    if (dd == 0) st_cells4(bPA, c + HD, mm, lv, 0.f, 0.f, fout);
                }
            }
            __syncthreads();                                                    // the combine buffers are free again
            continue;
        }

        // ================= a projection phase (or the logits) ========================================================================
        const int n_tiles = is_lm ? 1 : tiles_of(kind);
        const int u0 = is_lm ? 0 : first_tile(kind);
        if (u0 >= n_tiles) continue;
        // What the tile loop needs is worked out here, ahead of the polls, and pinned there: left to itself the compiler
        // puts these couple of hundred scalar instructions between the staging barrier and the first multiply, where they
        // are on the critical path (a wavefront issues one of them every four to five cycles).
        const int K = kind == PH_O ? nq : (kind == PH_DOWN ? ff : d), steps = K >> 5;
        const int wsh = kind == PH_GU ? 2 : 3;
        const int wv = kind == PH_GU ? (wave & 3) : wave;
        int s0 = (wv * steps) >> wsh, n = (((wv + 1) * steps) >> wsh) - s0;
        unsigned fout = step_flag(l, kind);
        int boff = plane_off(s0);
        asm volatile("" : "+s"(s0), "+s"(n), "+s"(fout), "+v"(boff));
        // the residual columns of the first tile (O, down: written two phases ago) are asked for ahead of the staging
        auto residual = [&](int u) -> float4 {
            const int c = u * 16 + 4 * lq;
            if (ph == PH_O) {                                                    // first layer: the residual is the embedding
                const uint2 e = *reinterpret_cast<const uint2*>(a.embed + (size_t)tok_row * d + c);
                return make_float4(__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xFFFF0000u),
                                   __uint_as_float(e.y << 16), __uint_as_float(e.y & 0xFFFF0000u));
            }
            return poll4(bX, xcopy + li * d + c, kind == PH_O ? step_flag(l - 1, PH_DOWN) : step_flag(l, PH_O));
        };
        float4 x_first = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!is_lm && (kind == PH_O || kind == PH_DOWN) && wave == 0 && row_ok) x_first = residual(u0);
        // ---- stage the input rows as planes in LDS ----
        if (is_lm || kind == PH_QKV || kind == PH_GU) {
            // RMSNorm by linearity: norm(x) W^T = r * ((gain . x) W^T) with r = rsqrt(mean(x^2) + eps) per row, so the planes
            // of gain . x are staged as soon as x is there and the row-wide sum only has to be ready for the epilogue, which
            // multiplies by r (first layer: x = the token embeddings, else the residual stream X as the phase before left it)
            const float* gain = is_lm ? a.final_norm : (kind == PH_QKV ? a.an[l] : a.fn[l]);
            const bool src_embed = (is_lm ? a.n_layers : ph) == 0;
            const unsigned fin = (is_lm || kind == PH_QKV) ? step_flag(l - 1, PH_DOWN) : step_flag(l, PH_O);
            const int n4 = M * d / 4;
            float ss0 = 0.f, ss1 = 0.f;
#pragma unroll
            for (int i = 0; i < STEP_XR; ++i) {
                const int g = tid + i * STEP_THREADS;
                if (g < n4) {
                    const int m = g * 4 >= d ? 1 : 0, c = g * 4 - m * d;
                    const float4 gn = *reinterpret_cast<const float4*>(gain + c);
                    float4 xv;
                    if (src_embed) {
                        const uint2 e = *reinterpret_cast<const uint2*>(a.embed + (size_t)a.tok[m] * d + c);
                        xv = make_float4(__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xFFFF0000u),
                                         __uint_as_float(e.y << 16), __uint_as_float(e.y & 0xFFFF0000u));
                    } else {
                        xv = poll4(bX, xcopy + g * 4, fin);
                    }
                    put_planes(m, c, xv.x * gn.x, xv.y * gn.y, xv.z * gn.z, xv.w * gn.w);
                    const float s = xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
                    if (m == 0) ss0 += s; else ss1 += s;
                }
            }
            ss0 = wsum(ss0); ss1 = wsum(ss1);
            if (lane == 0) { s_part[wave][0] = ss0; s_part[wave][1] = ss1; }      // read behind the staging barrier: row_scale()
        } else if (kind == PH_O) {
            // the attention output: every workgroup combines the key splits of the whole rows itself (a few KB).  Four
            // columns per item; the (max, sum) of up to four splits at a time, then their weighted partial outputs.
            const unsigned fin = step_flag(l, PH_ATT);
            const int per_row = nq / 4, items = M * per_row;
            for (int it = tid; it < items; it += STEP_THREADS) {
                const int m = it >= per_row ? 1 : 0, col = (it - m * per_row) * 4, h = col / HD, d0 = col & (HD - 1);
                const int Se = m == 0 ? Se_row0 : Se_row1;
                const int base = ((m * H + h) * (S + 1)) * PCELLS;
                float mm = -INFINITY, lsum = 0.f, o4[4] = {0.f, 0.f, 0.f, 0.f};
                for (int sx = 0; sx <= Se; sx += STEP_MB) {                            // the used splits, then the own keys' partial (slot S)
                    // (max, sum, pad, pad) of and the four output cells of up to STEP_MB partials in one round of loads
                    // (every cell of a used partial is written, also by a unit that had nothing to attend to)
                    int pc[2 * STEP_MB], slot[STEP_MB];
                    float4 pv_[2 * STEP_MB], ml[STEP_MB], ov[STEP_MB];
#pragma unroll
                    for (int q = 0; q < STEP_MB; ++q) slot[q] = sx + q < Se ? sx + q : (sx + q == Se ? S : -1);
#pragma unroll
                    for (int q = 0; q < STEP_MB; ++q) {
                        pc[2 * q] = slot[q] >= 0 ? base + slot[q] * PCELLS + HD : -1;
                        pc[2 * q + 1] = slot[q] >= 0 ? base + slot[q] * PCELLS + d0 : -1;
                    }
                    poll4n(bPA, pc, fin, pv_);
#pragma unroll
                    for (int q = 0; q < STEP_MB; ++q) { ml[q] = pv_[2 * q]; ov[q] = pv_[2 * q + 1]; }
                    float gm = mm;
#pragma unroll
                    for (int q = 0; q < STEP_MB; ++q)
                        if (slot[q] >= 0) gm = fmaxf(gm, ml[q].x);
                    if (gm == -INFINITY) continue;
                    const float keep = __expf(mm - gm);                         // 0 when nothing was accumulated yet
                    lsum *= keep;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] *= keep;
#pragma unroll
                    for (int q = 0; q < STEP_MB; ++q) {
                        const float ms = ml[q].x;
                        const float f = (slot[q] < 0 || ms == -INFINITY) ? 0.f : __expf(ms - gm);
                        if (f == 0.f) continue;
                        lsum += ml[q].y * f;
                        o4[0] += ov[q].x * f; o4[1] += ov[q].y * f; o4[2] += ov[q].z * f; o4[3] += ov[q].w * f;
                    }
                    mm = gm;
                }
                const float inv = lsum > 0.f ? __builtin_amdgcn_rcpf(lsum) : 0.f;
                put_planes(m, col, o4[0] * inv, o4[1] * inv, o4[2] * inv, o4[3] * inv);
            }
        } else {
            // SwiGLU output of the gate / up phase
            const unsigned fin = step_flag(l, PH_GU);
            const int per_row = ff / 4;
            int ac[STEP_XR];
            float4 av[STEP_XR];
#pragma unroll
            for (int i = 0; i < STEP_XR; ++i) ac[i] = tid + i * STEP_THREADS < M * per_row ? (tid + i * STEP_THREADS) * 4 : -1;
            poll4n(bACT, ac, fin, av);
#pragma unroll
            for (int i = 0; i < STEP_XR; ++i) {
                const int g = tid + i * STEP_THREADS;
                if (g < M * per_row) {
                    const int m = g >= per_row ? 1 : 0, c = (g - m * per_row) * 4;
                    put_planes(m, c, av[i].x, av[i].y, av[i].z, av[i].w);
                }
            }
        }
        if (!alive()) return;                                                    // the planes are in LDS (or somebody gave up)

        if (is_lm) {
            // ---- logits: a wavefront owns whole 16-row tiles of the vocabulary, no sharing of K ----
            const int steps_d = d >> 5;
            const int v_tiles = (a.V + 15) / 16;
            const float rs_row = row_scale(min(li, M - 1));
            for (int tw = wg * STEP_WAVES + wave; tw < v_tiles; tw += G * STEP_WAVES) {
                const uint32_t tile_off = step_tile_off(tw * 16 + li, d, lq);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                for (int sb = 0; sb < steps_d; sb += STEP_MAXS) {
                    const int nn = min(STEP_MAXS, steps_d - sb);
                    wfetch(a.lm_head, tile_off, sb, nn);
                    const f32x4 part = wmma(plane_off(sb), nn);
                    acc[0] += part[0]; acc[1] += part[1]; acc[2] += part[2]; acc[3] += part[3];
                }
                acc[0] *= rs_row; acc[1] *= rs_row; acc[2] *= rs_row; acc[3] *= rs_row;
                // lane holds D[column tw*16 + 4 lq + e][row li]; row m = b * q_len + j gets logits if j >= q_len - logit_rows
                if (row_ok) {
                    const int bq = li >> qs, j = li & qs, r = j - (q_len - a.logit_rows);
                    if (r >= 0) {
                        float* o = a.logits + (size_t)bq * a.logits_bstride + (size_t)r * a.V + tw * 16 + 4 * lq;
                        const int cb = tw * 16 + 4 * lq;
                        if (cb + 3 < a.V && (reinterpret_cast<uintptr_t>(o) & 15) == 0) {
                            *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (cb + e < a.V) o[e] = acc[e];
                        }
                    }
                }
            }
            break;
        }

        // ---- the workgroup's tiles ----
        // One tile per workgroup and phase (the host admits no model with more tiles than workgroups): its weights were
        // asked for at the top of an earlier phase.  A loop over further tiles here made the compiler carry a second copy
        // of the weight registers and the addresses of 16 more loads through every phase.
        {
            const int u = u0;
            const int c = u * 16 + 4 * lq;                                       // lane's four output columns (wavefront 0)
            // what the epilogue needs from memory is requested before the multiply
            float4 x_old = make_float4(0.f, 0.f, 0.f, 0.f);
            float2 rc0 = make_float2(1.f, 0.f), rc1 = make_float2(1.f, 0.f);
            if (wave == 0 && row_ok) {
                if (kind == PH_O || kind == PH_DOWN) {
                    x_old = x_first;
                } else if (kind == PH_QKV && c < nq + nkv) {
                    const int hc = c & (HD - 1);
                    rc0 = a.rope[(size_t)m_row * (HD / 2) + hc / 2];
                    rc1 = a.rope[(size_t)m_row * (HD / 2) + hc / 2 + 1];
                }
            }
            const f32x4 acc = wmma(boff, n);
            // red[] is free: whoever read it last did so before the workgroup-wide check that ended its phase
            *reinterpret_cast<f32x4*>(&red[wave][lane * 4]) = acc;
            __syncthreads();
            if (wave == 0 && row_ok) {
                // all eight shares are read at once (a loop up to a run-time count reads them one LDS round trip after the
                // other); gate / up: the first four wavefronts hold the gate columns, the last four the up columns
                f32x4 pw[STEP_WAVES];
#pragma unroll
                for (int v = 0; v < STEP_WAVES; ++v) pw[v] = *reinterpret_cast<const f32x4*>(&red[v][lane * 4]);
                f32x4 t, t2;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    t[e] = (pw[0][e] + pw[1][e]) + (pw[2][e] + pw[3][e]);
                    t2[e] = (pw[4][e] + pw[5][e]) + (pw[6][e] + pw[7][e]);
                }
                if (kind != PH_GU) { t[0] += t2[0]; t[1] += t2[1]; t[2] += t2[2]; t[3] += t2[3]; }
                if (kind == PH_QKV || kind == PH_GU) {                           // the deferred RMS scale of the input row
                    const float rs = row_scale(li);
                    t[0] *= rs; t[1] *= rs; t[2] *= rs; t[3] *= rs;
                }
                if (kind == PH_GU) {
                    const float rs = row_scale(li);
                    float h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = t[e] * __builtin_amdgcn_rcpf(1.0f + __expf(-t[e])) * (t2[e] * rs);
                    st_cells4(bACT, li * ff + c, h[0], h[1], h[2], h[3], fout);
                } else if (kind == PH_O || kind == PH_DOWN) {
#pragma unroll
                    for (int cp = 0; cp < STEP_XCOPIES; ++cp)
                        st_cells4(bX, cp * (M * d) + li * d + c, x_old.x + t[0], x_old.y + t[1], x_old.z + t[2], x_old.w + t[3], fout);
                } else if (c < nq + nkv) {
                    const int hc = c & (HD - 1);
                    const float r0 = t[0] * rc0.x - t[1] * rc0.y, r1 = t[0] * rc0.y + t[1] * rc0.x;
                    const float r2 = t[2] * rc1.x - t[3] * rc1.y, r3 = t[2] * rc1.y + t[3] * rc1.x;
                    if (c < nq) {
                        st_cells4(bQ, li * nq + c, r0, r1, r2, r3, fout);
                    } else {
                        // the key as the cache holds it (bf16); the attention phase of this pass takes it from the
                        // exchange buffer, later passes from the cache
                        const uint32_t w0 = pack_bf16(r0, r1), w1 = pack_bf16(r2, r3);
                        st_cells4(bKVN, li * 2 * nkv + (c - nq), __uint_as_float(w0 << 16), __uint_as_float(w0 & 0xFFFF0000u),
                                  __uint_as_float(w1 << 16), __uint_as_float(w1 & 0xFFFF0000u), fout);
                        if (p_row >= 0) {
                            const int kh = (c - nq) / HD;
                            uint16_t* dst = reinterpret_cast<uint16_t*>(kc) + (((size_t)b_row * KVH + kh) * a.cache_len + p_row) * HD + hc;
                            *reinterpret_cast<uint2*>(dst) = make_uint2(w0, w1);
                        }
                    }
                } else {
                    const int cv = c - nq - nkv;
                    const uint32_t w0 = pack_bf16(t[0], t[1]), w1 = pack_bf16(t[2], t[3]);
                    st_cells4(bKVN, li * 2 * nkv + nkv + cv, __uint_as_float(w0 << 16), __uint_as_float(w0 & 0xFFFF0000u),
                              __uint_as_float(w1 << 16), __uint_as_float(w1 & 0xFFFF0000u), fout);
                    if (p_row >= 0) {
                        const int vh = cv / HD, hc = cv & (HD - 1);
                        uint16_t* base = reinterpret_cast<uint16_t*>(vc) + ((size_t)b_row * KVH + vh) * (size_t)a.cache_len * HD;
                        base[v_index<uint16_t>(p_row, hc, HD)] = (uint16_t)(w0 & 0xFFFFu);
                        base[v_index<uint16_t>(p_row, hc + 1, HD)] = (uint16_t)(w0 >> 16);
                        base[v_index<uint16_t>(p_row, hc + 2, HD)] = (uint16_t)(w1 & 0xFFFFu);
                        base[v_index<uint16_t>(p_row, hc + 3, HD)] = (uint16_t)(w1 >> 16);
                    }
                }
            }
        }
        if (!alive()) return;                    // the planes and red[] are free again; a poll of the epilogue may have given up
        next_own(ph + 1);                        // fetched at the top of the next phase
    }
}

// ---- host side --------------------------------------------------------------------------------------------------
static size_t step_lds_bytes(int M, int d, int nq, int ff, int hd, int R) {
    const int kmax = d > nq ? (d > ff ? d : ff) : (nq > ff ? nq : ff);
    const size_t planes = (size_t)2 * M * (kmax + 8) * 2;
    const size_t att = ((size_t)2 * STEP_WAVES * 16 + (size_t)STEP_WAVES * R * (hd + 1)) * 4 + (size_t)2 * (hd / 32) * 64 * 16;
    return planes > att ? planes : att;
}

bool step_fits(const bs_model_cfg& c, int B, int q_len, int n_layers) {
    const int M = B * q_len, nq = c.n_heads * c.head_dim, nkv = c.n_kv_heads * c.head_dim;
    if (M < 1 || M > 2 || q_len > 2 || n_layers > STEP_MAXL) return false;
    // head dimension 128 needs twice the registers for the keys, values and queries in flight and spills; a vocabulary of
    // more than about one and a half 16-row tiles per wavefront leaves the logits phase waiting for one tile after the
    // other (measured, 4 layers x 1024 wide, 128 heads, 128256 tokens: 340 us against 190 us of the kernel-per-phase path)
    if (c.head_dim != 64 || c.vocab > 3 * 16 * STEP_WAVES * step_grid() / 2) return false;
    if (c.d_model % 32 || nq % 32 || c.d_ff % 32 || nkv % 16) return false;
    const int grid = step_grid();
    if ((nq + 2 * nkv) / 16 > grid || c.d_ff / 16 > grid || c.d_model / 16 > grid) return false;   // one tile per workgroup and phase
    const int R = c.n_heads / c.n_kv_heads * q_len;
    if (R > 16) return false;
    auto share = [](int K, int waves) { return (K / 32 + waves - 1) / waves; };     // k steps per wavefront
    if (share(c.d_model, STEP_WAVES / 2) > STEP_MAXS || share(nq, STEP_WAVES) > STEP_MAXS || share(c.d_ff, STEP_WAVES) > STEP_MAXS) return false;
    if ((size_t)M * c.d_model / 4 > (size_t)STEP_XR * STEP_THREADS) return false;   // the staged rows are held in registers
    if ((double)M * c.n_heads * 64.0 * (c.head_dim + 4) * 8.0 > 2.0e9) return false; // 32-bit byte offsets into the exchange buffers
    return step_lds_bytes(M, c.d_model, nq, c.d_ff, c.head_dim, R) <= 56 * 1024;
}

int step_splits(const bs_model_cfg& c, int B, int max_len) {
    const int G = step_grid();
    const int room = G / (B * c.n_kv_heads) - 1;                 // one unit per (sequence, kv head) takes the own keys
    const int blocks = (max_len + 31) / 32;
    int s = (blocks + STEP_WAVES * STEP_BLK - 1) / (STEP_WAVES * STEP_BLK);
    if (s > 16) s = 16;                                          // longer caches: a wavefront walks several blocks
    if (s > room) s = room;
    return s < 1 ? 0 : s;
}

size_t step_exchange_bytes(const bs_model_cfg& c, int M, int splits, size_t off[5]) {
    const size_t nq = (size_t)c.n_heads * c.head_dim, nkv = (size_t)c.n_kv_heads * c.head_dim;
    const size_t cells[5] = {(size_t)STEP_XCOPIES * M * c.d_model, (size_t)M * nq, (size_t)M * 2 * nkv,
                             (size_t)M * c.n_heads * (splits + 1) * (c.head_dim + 4), (size_t)M * c.d_ff};
    size_t total = 0;
    for (int i = 0; i < 5; ++i) {
        if (off) off[i] = total;
        total += align_up(cells[i] * 8, 256);
    }
    return total;
}

int step_grid() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&p, dev) != hipSuccess) return 0;
        cus = p.multiProcessorCount;
    }
    return cus;
}

int launch_step(const StepArgs& a_in, hipStream_t s) {
    StepArgs a = a_in;
    const int nq = a.H * a.hd;
    const int R = a.H / a.KVH * a.q_len;
    const int kmax = a.d > nq ? (a.d > a.ff ? a.d : a.ff) : (nq > a.ff ? nq : a.ff);
    a.kp = kmax + 8;
    const int G = step_grid();
    BS_REQUIRE(G >= 8, BS_EHIP, "step: cannot read the number of compute units");
    BS_REQUIRE(a.splits >= 1 && a.B * a.KVH * (a.splits + 1) <= G, BS_ESHAPE, "step: %d attention units exceed the %d resident workgroups",
               a.B * a.KVH * (a.splits + 1), G);
    const size_t lds = step_lds_bytes(a.M, a.d, nq, a.ff, a.hd, R);
    BS_REQUIRE(lds <= 56 * 1024, BS_ESHAPE, "step: %zu bytes of LDS", lds);
    // one workgroup per compute unit: all of them are resident together, which the polling of the exchange cells relies on
    BS_REQUIRE(a.hd == 64, BS_ESHAPE, "step: head dimension %d", a.hd);
    hipLaunchKernelGGL((dec_step_kernel<64>), dim3(G), dim3(STEP_THREADS), lds, s, a);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

}  // namespace bs
