// Host side of the model path: handles, workspace carving, the forward pass schedule (verification
// pass of App. A and the draft steps), prompt prefill, and the round driver (Alg. 2 with vanilla
// speculative decoding; one iteration of the loop of Alg. 3 on the device).
#include <atomic>
#include <new>
#include <vector>
#include "common.h"
#include "kernels.h"
#include "sample.h"

using namespace bs;

// polls of one exchange cell before a resident step gives up: about a quarter of a second at the default
constexpr unsigned STEP_DEFAULT_POLLS = 1u << 18;
static std::atomic<unsigned> g_step_polls{STEP_DEFAULT_POLLS};

struct bs_model {
    bs_model_cfg cfg;
    const void* embed;
    const float* final_norm;
    const void* lm_head;
    std::vector<bs_layer_weights> layers;   // projections point into the packed copy once bs_model_pack has run
    bool packed = false;
};

struct bs_kv {
    bs_model_cfg cfg;
    int B, max_len;
    char* buf;
    size_t bytes;
};

static size_t esize(int dtype) { return dtype == BS_BF16 ? 2 : 4; }
static int cache_rows(int max_len) { return (max_len + 31) / 32 * 32; }   // V is stored in blocks of 32 keys

static int check_cfg(const bs_model_cfg* c, const char* who) {
    BS_REQUIRE(c, BS_EINVAL, "%s: cfg is NULL", who);
    BS_REQUIRE(c->dtype == BS_F32 || c->dtype == BS_BF16, BS_EDTYPE, "%s: dtype %d", who, c->dtype);
    BS_REQUIRE(c->n_layers >= 1 && c->d_model >= 8 && c->n_heads >= 1 && c->n_kv_heads >= 1 && c->d_ff >= 8 && c->vocab >= 1,
               BS_ESHAPE, "%s: non-positive model dimension", who);
    BS_REQUIRE(c->n_heads % c->n_kv_heads == 0, BS_ESHAPE, "%s: n_heads %d not a multiple of n_kv_heads %d", who, c->n_heads, c->n_kv_heads);
    BS_REQUIRE(c->head_dim % 8 == 0 && c->head_dim >= 8 && c->head_dim <= 128, BS_ESHAPE,
               "%s: head_dim %d must be a multiple of 8 in [8,128]", who, c->head_dim);
    BS_REQUIRE(c->dtype != BS_BF16 || c->head_dim == 64 || c->head_dim == 128, BS_ESHAPE,
               "%s: bf16 models need head_dim 64 or 128 (MFMA attention), got %d", who, c->head_dim);
    BS_REQUIRE(c->d_model % 8 == 0 && c->d_ff % 8 == 0, BS_ESHAPE, "%s: d_model and d_ff must be multiples of 8", who);
    BS_REQUIRE(c->vocab <= (1 << 20), BS_ESHAPE, "%s: vocab %d > 2^20", who, c->vocab);
    BS_REQUIRE(c->rope_base > 1.f && c->norm_eps > 0.f, BS_EINVAL, "%s: rope_base/norm_eps out of range", who);
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_model_create(const bs_model_cfg* cfg, const bs_model_weights* w, bs_model** out) {
    int rc = check_cfg(cfg, "bs_model_create");
    if (rc != BS_OK) return rc;
    BS_REQUIRE(w && out, BS_EINVAL, "bs_model_create: NULL argument");
    BS_REQUIRE(w->embed && w->final_norm && w->lm_head && w->layers, BS_EINVAL, "bs_model_create: NULL weight pointer");
    bs_model* m = new (std::nothrow) bs_model();
    BS_REQUIRE(m, BS_EINVAL, "bs_model_create: out of host memory");
    m->cfg = *cfg; m->embed = w->embed; m->final_norm = w->final_norm; m->lm_head = w->lm_head;
    m->layers.assign(w->layers, w->layers + cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
        const bs_layer_weights& L = m->layers[l];
        const void* ptrs[9] = {L.attn_norm, L.wq, L.wk, L.wv, L.wo, L.ffn_norm, L.w_gate, L.w_up, L.w_down};
        for (int i = 0; i < 9; ++i) {
            if (!ptrs[i] || (reinterpret_cast<uintptr_t>(ptrs[i]) & 15)) {
                delete m;
                BS_FAIL(BS_EINVAL, "bs_model_create: layer %d weight %d is NULL or not 16-byte aligned", l, i);
            }
        }
    }
    *out = m;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_model_destroy(bs_model* m) { delete m; return BS_OK; }

// ---- tiled copy of the projection matrices -----------------------------------------------------------
static bool packable(const bs_model_cfg& c) {
    const int nq = c.n_heads * c.head_dim, nkv = c.n_kv_heads * c.head_dim;
    return c.dtype == BS_BF16 && c.d_model % 32 == 0 && nq % 32 == 0 && c.d_ff % 32 == 0 && nq % 16 == 0 && nkv % 16 == 0 && c.d_ff % 16 == 0;
}

extern "C" __attribute__((visibility("default"))) size_t bs_model_packed_bytes(const bs_model_cfg* c) {
    if (!c || !packable(*c)) return 0;
    const int nq = c->n_heads * c->head_dim, nkv = c->n_kv_heads * c->head_dim;
    size_t per_layer = 0;
    auto add = [&](int N, int K) { per_layer += align_up(packed_elems(N, K) * 2, 256); };
    add(nq, c->d_model); add(nkv, c->d_model); add(nkv, c->d_model); add(c->d_model, nq);
    add(c->d_ff, c->d_model); add(c->d_ff, c->d_model); add(c->d_model, c->d_ff);
    return per_layer * c->n_layers + align_up(packed_elems(c->vocab, c->d_model) * 2, 256);
}

extern "C" __attribute__((visibility("default"))) int bs_model_pack(bs_model* m, void* dev_buf, size_t bytes, void* stream) {
    BS_REQUIRE(m && dev_buf, BS_EINVAL, "bs_model_pack: NULL argument");
    BS_REQUIRE(!m->packed, BS_ESTATE, "bs_model_pack: model is already packed");
    const bs_model_cfg& c = m->cfg;
    const size_t need = bs_model_packed_bytes(&c);
    BS_REQUIRE(need > 0, BS_ESHAPE, "bs_model_pack: needs a bf16 model whose d_model, n_heads*head_dim and d_ff are multiples of 32 "
                                    "and whose n_kv_heads*head_dim is a multiple of 16");
    BS_REQUIRE(bytes >= need, BS_EWORKSPACE, "bs_model_pack: buffer %zu < %zu bytes", bytes, need);
    BS_REQUIRE((reinterpret_cast<uintptr_t>(dev_buf) & 255) == 0, BS_EWORKSPACE, "bs_model_pack: buffer not 256-byte aligned");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const int nq = c.n_heads * c.head_dim, nkv = c.n_kv_heads * c.head_dim;
    char* cur = reinterpret_cast<char*>(dev_buf);
    int rc = BS_OK;
    auto pack = [&](const void*& w, int N, int K) {
        if (rc != BS_OK) return;
        rc = launch_pack_weights(w, cur, N, K, s);
        w = cur;
        cur += align_up(packed_elems(N, K) * 2, 256);
    };
    std::vector<bs_layer_weights> layers = m->layers;
    const void* head = m->lm_head;
    for (bs_layer_weights& L : layers) {
        pack(L.wq, nq, c.d_model); pack(L.wk, nkv, c.d_model); pack(L.wv, nkv, c.d_model); pack(L.wo, c.d_model, nq);
        pack(L.w_gate, c.d_ff, c.d_model); pack(L.w_up, c.d_ff, c.d_model); pack(L.w_down, c.d_model, c.d_ff);
    }
    pack(head, c.vocab, c.d_model);
    if (rc != BS_OK) return rc;
    m->layers = layers; m->lm_head = head; m->packed = true;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) size_t bs_kv_bytes(const bs_model_cfg* c, int B, int max_len) {
    if (!c || B < 1 || max_len < 1) return 0;
    return (size_t)c->n_layers * 2 * B * c->n_kv_heads * (size_t)cache_rows(max_len) * c->head_dim * esize(c->dtype);
}

extern "C" __attribute__((visibility("default"))) int bs_kv_bind(const bs_model* m, int B, int max_len, void* dev_buf, size_t bytes, bs_kv** out) {
    BS_REQUIRE(m && dev_buf && out, BS_EINVAL, "bs_kv_bind: NULL argument");
    BS_REQUIRE(B >= 1 && max_len >= 1, BS_ESHAPE, "bs_kv_bind: B=%d max_len=%d", B, max_len);
    BS_REQUIRE(bytes >= bs_kv_bytes(&m->cfg, B, max_len), BS_EWORKSPACE, "bs_kv_bind: buffer %zu < %zu bytes", bytes, bs_kv_bytes(&m->cfg, B, max_len));
    BS_REQUIRE((reinterpret_cast<uintptr_t>(dev_buf) & 255) == 0, BS_EWORKSPACE, "bs_kv_bind: buffer not 256-byte aligned");
    bs_kv* kv = new (std::nothrow) bs_kv();
    BS_REQUIRE(kv, BS_EINVAL, "bs_kv_bind: out of host memory");
    kv->cfg = m->cfg; kv->B = B; kv->max_len = max_len; kv->buf = reinterpret_cast<char*>(dev_buf); kv->bytes = bytes;
    *out = kv;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_kv_destroy(bs_kv* kv) { delete kv; return BS_OK; }

// ---- forward workspace ----------------------------------------------------------------------------
static int attn_splits(int B, int H, int max_len) {
    int by_len = (max_len + 511) / 512;              // about four 32-key blocks per wavefront at full length (measured: 5.7 ms per round against 6.1 with one block each; 256..1024 keys per split are within 2 %)
    int by_fill = (1024 + B * H - 1) / (B * H);      // enough workgroups to cover 256 CUs a few times
    int s = by_len < by_fill ? by_len : by_fill;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return s;
}

struct FwdWs {
    int32_t* status; int32_t* pos; int32_t* tok; float2* rope; float* x; void* h; float* q; void* att; void* act; float* ssq;
    char* xch; size_t xch_bytes;    // resident step kernel: exchange cells (one or two rows only)
    char* acells; size_t acells_bytes;   // attention: exchange cells of the key splits (up to 16 rows of a bf16 model)
    float *part_qkv, *part_o, *part_gu, *part_d, *part_attn;
    int ks_qkv, ks_o, ks_gu, ks_d;
    size_t total;
};

// Activations take 4 bytes per element in either dtype: float, or a bf16 (hi, lo) pair of planes.
static FwdWs carve(const bs_model_cfg& c, int B, int q_len, int max_len, char* base) {
    FwdWs w;
    const size_t M = (size_t)B * q_len;
    const size_t Mp = M < 16 ? 16 : M;           // planes in the 16-row tiled layout of the whole-K projections
    const size_t nq = (size_t)c.n_heads * c.head_dim, nkv = (size_t)c.n_kv_heads * c.head_dim;
    w.ks_qkv = gemm_splits(c.dtype, (int)(nq + 2 * nkv), c.d_model, (int)M);
    w.ks_o = gemm_splits(c.dtype, c.d_model, (int)nq, (int)M);
    w.ks_gu = gemm_splits(c.dtype, 2 * c.d_ff, c.d_model, (int)M);
    w.ks_d = gemm_splits(c.dtype, c.d_model, c.d_ff, (int)M);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return base ? base + o : (char*)nullptr; };
    w.status = (int32_t*)take(256);
    w.pos = (int32_t*)take(M * 4);
    w.tok = (int32_t*)take(M * 4);
    w.rope = (float2*)take(M * (c.head_dim / 2) * 8);
    w.x = (float*)take(M * c.d_model * 4);
    w.h = take(Mp * c.d_model * 4);
    w.q = (float*)take(M * nq * 4);
    w.att = take(Mp * nq * 4);
    w.act = take(Mp * c.d_ff * 4);
    w.ssq = (float*)take(M * (c.d_model / 16 + 1) * 4);
    w.xch_bytes = (M <= 2 && step_splits(c, B, max_len) > 0) ? step_exchange_bytes(c, (int)M, step_splits(c, B, max_len), nullptr) : 0;
    w.xch = take(w.xch_bytes);
    w.acells_bytes = (c.dtype == BS_BF16 && M <= 16 && M > 2) ? attn_cells_bytes((int)M, c.n_heads, c.head_dim, attn_splits(B, c.n_heads, max_len)) : 0;
    w.acells = take(w.acells_bytes);
    w.part_qkv = (float*)take(M * (nq + 2 * nkv) * 4 * w.ks_qkv);
    w.part_o = (float*)take(M * c.d_model * 4 * w.ks_o);
    w.part_gu = (float*)take(M * 2 * c.d_ff * 4 * w.ks_gu);
    w.part_d = (float*)take(M * c.d_model * 4 * w.ks_d);
    w.part_attn = (float*)take(M * c.n_heads * attn_splits(B, c.n_heads, max_len) * (size_t)(c.head_dim + 4) * 4);
    w.total = off;
    return w;
}

// The split-K factors depend on the row count, so the need is not monotone in q_len: take the largest.
static size_t carve_max(const bs_model_cfg& c, int B, int max_q_len, int max_len) {
    size_t need = 0;
    for (int q = 1; q <= max_q_len; ++q) {
        const size_t t = carve(c, B, q, max_len, nullptr).total;
        if (t > need) need = t;
    }
    return need;
}

extern "C" __attribute__((visibility("default"))) size_t bs_forward_workspace_bytes(const bs_model_cfg* c, int B, int max_q_len, int max_len) {
    if (!c || B < 1 || max_q_len < 1 || max_len < 1) return 0;
    return carve_max(*c, B, max_q_len, max_len);
}

// One pass of the model over q_len tokens per sequence (see bs_verify_forward).  kv position of query j is
// kv_len[b] + kv_base + j; logits of the trailing logit_rows rows go to logits + b*logits_bstride + r*V.
static int forward(const bs_model* m, const bs_kv* kv, const int32_t* q_tokens, int q_stride, const int32_t* kv_len,
                   int kv_base, int q_len, int logit_rows, float* logits, size_t logits_bstride, void* ws, size_t ws_bytes,
                   hipStream_t s) {
    const bs_model_cfg& c = m->cfg;
    const int B = kv->B, M = B * q_len, dt = c.dtype;
    const size_t need = carve(c, B, q_len, kv->max_len, nullptr).total;
    BS_REQUIRE(ws_bytes >= need, BS_EWORKSPACE, "forward: workspace %zu < %zu bytes", ws_bytes, need);
    BS_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255) == 0, BS_EWORKSPACE, "forward: workspace not 256-byte aligned");
    FwdWs w = carve(c, B, q_len, kv->max_len, reinterpret_cast<char*>(ws));
    const int H = c.n_heads, KVH = c.n_kv_heads, hd = c.head_dim, d = c.d_model, ff = c.d_ff;
    const int nq = H * hd, nkv = KVH * hd, nqkv = nq + 2 * nkv;
    const size_t es = esize(dt);
    const int crow = cache_rows(kv->max_len);
    const size_t kv_layer = (size_t)2 * B * KVH * (size_t)crow * hd * es;
    const int splits = attn_splits(B, H, kv->max_len);
    int rc;
#define BS_TRY(expr) do { rc = (expr); if (rc != BS_OK) return rc; } while (0)
    const float* pend = nullptr;      // split-K partials of the last residual projection, not yet added to x
    // A handful of rows (draft steps): fused schedule, 5 kernels per layer; needs the tiled weights.
    const bool few_rows = dt == BS_BF16 && m->packed && gemm_dec_fits(M, d) && gemm_dec_fits(M, nq) && gemm_dec_fits(M, ff);
    // One or two rows of a small model: one resident kernel for the whole pass.
    const int st_splits = M <= 2 ? step_splits(c, B, kv->max_len) : 0;
    const bool resident = few_rows && st_splits > 0 && step_fits(c, B, q_len, c.n_layers);
    BS_TRY(launch_prep(q_tokens, q_stride, kv_len, kv_base, B, q_len, kv->max_len, c.vocab, hd, c.rope_base, w.pos, w.tok,
                       w.rope, w.status, resident ? w.xch : w.acells_bytes ? w.acells : nullptr, resident ? w.xch_bytes : w.acells_bytes, s));
    if (resident) {
        StepArgs a = {};
        for (int l = 0; l < c.n_layers; ++l) {
            const bs_layer_weights& L = m->layers[l];
            const void* ptrs[7] = {L.wq, L.wk, L.wv, L.wo, L.w_gate, L.w_up, L.w_down};
            for (int i = 0; i < 7; ++i) a.w[l][i] = reinterpret_cast<const uint16_t*>(ptrs[i]);
            a.an[l] = L.attn_norm; a.fn[l] = L.ffn_norm;
        }
        a.embed = reinterpret_cast<const uint16_t*>(m->embed); a.final_norm = m->final_norm;
        a.lm_head = reinterpret_cast<const uint16_t*>(m->lm_head);
        a.n_layers = c.n_layers; a.d = d; a.H = H; a.KVH = KVH; a.hd = hd; a.ff = ff; a.V = c.vocab; a.eps = c.norm_eps;
        a.B = B; a.q_len = q_len; a.M = M; a.logit_rows = logit_rows;
        a.pos = w.pos; a.tok = w.tok; a.rope = w.rope;
        a.kv = kv->buf; a.kv_layer = kv_layer; a.cache_len = crow;
        size_t off[5];
        step_exchange_bytes(c, M, st_splits, off);
        a.X = w.xch + off[0]; a.Q = w.xch + off[1]; a.KVN = w.xch + off[2]; a.PA = w.xch + off[3]; a.ACT = w.xch + off[4];
        a.status = w.status; a.splits = st_splits;
        a.logits = logits; a.logits_bstride = logits_bstride;
        a.spin_limit = g_step_polls.load();       // polls of a cell before the pass is given up (status bit 16)
        BS_TRY(launch_step(a, s));
        return BS_OK;
    }
    if (few_rows) {
        const size_t pd = (size_t)M * d;
        uint16_t* hp = reinterpret_cast<uint16_t*>(w.h);
        BS_TRY(launch_embed_dec(w.tok, m->embed, m->layers[0].attn_norm, M, d, w.x, hp, pd, w.ssq, s));
        int ssq_tiles = 1;
        for (int l = 0; l < c.n_layers; ++l) {
            const bs_layer_weights& L = m->layers[l];
            char* kc = kv->buf + (size_t)l * kv_layer;
            char* vc = kc + kv_layer / 2;
            DecArgs a = {};
            a.xh = hp; a.x_plane = pd; a.w[0] = L.wq; a.w[1] = L.wk; a.w[2] = L.wv; a.seg_rows[0] = nq; a.seg_rows[1] = nkv;
            a.M = M; a.N = nqkv; a.K = d; a.ssq_in = w.ssq; a.ssq_tiles = ssq_tiles; a.eps = c.norm_eps;
            a.pos = w.pos; a.rope = w.rope; a.q_len = q_len; a.H = H; a.KVH = KVH; a.hd = hd; a.cache_len = crow;
            a.q_out = w.q; a.k_cache = reinterpret_cast<uint16_t*>(kc); a.v_cache = reinterpret_cast<uint16_t*>(vc);
            BS_TRY(launch_gemm_dec(EPI_QKV, a, s));
            BS_TRY(launch_attention(dt, w.q, kc, vc, w.pos, B, q_len, H, KVH, hd, crow, splits, w.part_attn,
                                    (size_t)M * nq, nullptr, false, nullptr, s));   // splits are merged by the O projection
            a = DecArgs{};
            a.att_part = w.part_attn; a.att_splits = splits; a.H = H; a.hd = hd;
            a.xh = reinterpret_cast<const uint16_t*>(w.att); a.x_plane = (size_t)M * nq; a.w[0] = L.wo; a.M = M; a.N = d; a.K = nq;
            a.x = w.x; a.gain_next = L.ffn_norm; a.out_planes = hp; a.out_plane = pd; a.ssq_out = w.ssq;
            BS_TRY(launch_gemm_dec(EPI_RESID, a, s));
            ssq_tiles = d / 16;
            a = DecArgs{};
            a.xh = hp; a.x_plane = pd; a.w[0] = L.w_gate; a.w[1] = L.w_up; a.M = M; a.N = ff; a.K = d;
            a.ssq_in = w.ssq; a.ssq_tiles = ssq_tiles; a.eps = c.norm_eps;
            a.out_planes = reinterpret_cast<uint16_t*>(w.act); a.out_plane = (size_t)M * ff;
            BS_TRY(launch_gemm_dec(EPI_SWIGLU, a, s));
            const bool more = l + 1 < c.n_layers;
            a = DecArgs{};
            a.xh = reinterpret_cast<const uint16_t*>(w.act); a.x_plane = (size_t)M * ff; a.w[0] = L.w_down; a.M = M; a.N = d; a.K = ff;
            a.x = w.x; a.gain_next = more ? m->layers[l + 1].attn_norm : nullptr; a.out_planes = hp; a.out_plane = pd;
            a.ssq_out = more ? w.ssq : nullptr;
            BS_TRY(launch_gemm_dec(EPI_RESID, a, s));
        }
    } else {
    // Up to 16 rows of a wide model (verification of one sequence): whole-K projections with the consumer's work in the
    // epilogue (gemm_rows_kernel), where the 16-column units of a projection fill at least four fifths of the compute units'
    // turns: QKV and gate/up from two units per compute unit on; O and down (one unit each on the 7B shape) only between
    // those two, which produce and consume the layouts they use.  A layer is then 6 kernels instead of 10.
    bool fuse_qkv = false, fuse_gu = false, fuse_o = false, fuse_d = false;
    if (dt == BS_BF16 && m->packed && M <= 16) {
        int g = 0;
        int tu = (hd == 64 || hd == 128) && nq % 16 == 0 && nkv % 16 == 0 ? gemm_rows_units(EPI_QKV, M, nqkv, d, &g) : 0;
        fuse_qkv = tu >= 2 && (nqkv / 16) * 5 >= g * tu * 4;
        tu = gemm_rows_units(EPI_SWIGLU, M, ff, d, &g);
        fuse_gu = tu >= 2 && (ff / 16) * 5 >= g * tu * 4;
        tu = gemm_rows_units(EPI_RESID, M, d, nq, &g);
        const bool wide = tu >= 1 && (d / 16) * 5 >= step_grid() * tu * 4;
        fuse_o = wide && fuse_gu && splits > 1 && nq % 32 == 0;
        fuse_d = wide && fuse_gu && fuse_qkv && gemm_rows_units(EPI_RESID, M, d, ff, &g) >= 1;
    }
    const int ssq_chunks = norm_chunks(d);
    // the attention's key splits combined inside its kernel (exchange cells, cleared by the prep kernel above)
    const bool in_kernel_merge = w.acells_bytes > 0 && splits > 1 && c.n_layers < 65536;
    AttnCells ac = {w.acells, w.acells_bytes, 0u, g_step_polls.load(), w.status};
    BS_TRY(launch_embed(dt, w.tok, m->embed, M, d, w.x, s));
    for (int l = 0; l < c.n_layers; ++l) {
        const bs_layer_weights& L = m->layers[l];
        char* kc = kv->buf + (size_t)l * kv_layer;
        char* vc = kc + kv_layer / 2;
        ac.flag = (unsigned)l + 1u;
        const bool defer = dt == BS_BF16;        // bf16: RMS scale applied behind the projection (see resid_sum_kernel)
        const float* ssq = defer ? w.ssq : nullptr;
        if (defer && fuse_d && l > 0) {}         // the down projection of the layer before left x, the planes and the sums of squares
        else if (defer)
            BS_TRY(launch_resid_sum(w.x, pend, w.ks_d, (size_t)M * d, L.attn_norm, d, M, fuse_qkv ? (size_t)16 * d : (size_t)M * d, w.h, w.ssq,
                                    fuse_qkv, s));
        else
            BS_TRY(launch_rmsnorm(dt, w.x, pend, w.ks_d, (size_t)M * d, L.attn_norm, d, c.norm_eps, B, q_len, q_len,
                                  (size_t)M * d, w.h, s));
        GemmArgs g;
        g.tiled = m->packed ? 1 : 0;
        g.x = w.h; g.x_plane = (size_t)M * d; g.w[0] = L.wq; g.w[1] = L.wk; g.w[2] = L.wv; g.seg_rows[0] = nq; g.seg_rows[1] = nkv;
        g.out = w.part_qkv; g.ks_stride = (size_t)M * nqkv; g.M = M; g.N = nqkv; g.K = d; g.ldo = nqkv; g.KS = w.ks_qkv;
        if (fuse_qkv) {
            DecArgs a = {};
            a.xh = reinterpret_cast<const uint16_t*>(w.h); a.x_plane = (size_t)16 * d; a.w[0] = L.wq; a.w[1] = L.wk; a.w[2] = L.wv;
            a.seg_rows[0] = nq; a.seg_rows[1] = nkv; a.M = M; a.N = nqkv; a.K = d;
            a.ssq_in = w.ssq; a.ssq_tiles = fuse_d && l > 0 ? d / 16 : ssq_chunks; a.eps = c.norm_eps;
            a.pos = w.pos; a.rope = w.rope; a.q_len = q_len; a.H = H; a.KVH = KVH; a.hd = hd; a.cache_len = crow;
            a.q_out = w.q; a.k_cache = reinterpret_cast<uint16_t*>(kc); a.v_cache = reinterpret_cast<uint16_t*>(vc);
            BS_TRY(launch_gemm_rows(EPI_QKV, a, s));
        } else {
        BS_TRY(launch_gemm(dt, g, s));
        BS_TRY(launch_rope_kv(dt, w.part_qkv, w.ks_qkv, (size_t)M * nqkv, w.pos, w.rope, M, q_len, H, KVH, hd, crow,
                              w.q, kc, vc, ssq, d, c.norm_eps, s));
        }
        BS_TRY(launch_attention(dt, w.q, kc, vc, w.pos, B, q_len, H, KVH, hd, crow, splits, w.part_attn,
                                fuse_o ? (size_t)16 * nq : (size_t)M * nq, w.att, fuse_o, in_kernel_merge ? &ac : nullptr, s));
        g.x = w.att; g.x_plane = (size_t)M * nq; g.w[0] = L.wo; g.w[1] = g.w[2] = nullptr; g.seg_rows[0] = d; g.seg_rows[1] = 0;
        g.out = w.part_o; g.ks_stride = (size_t)M * d; g.M = M; g.N = d; g.K = nq; g.ldo = d; g.KS = w.ks_o;
        if (fuse_o) {
            DecArgs a = {};
            a.xh = reinterpret_cast<const uint16_t*>(w.att); a.x_plane = (size_t)16 * nq; a.w[0] = L.wo; a.M = M; a.N = d; a.K = nq;
            a.x = w.x; a.gain_next = L.ffn_norm; a.out_planes = reinterpret_cast<uint16_t*>(w.h); a.out_plane = (size_t)16 * d; a.out_tiled = 1;
            a.ssq_out = w.ssq;
            BS_TRY(launch_gemm_rows(EPI_RESID, a, s));
        } else {
        BS_TRY(launch_gemm(dt, g, s));
        if (defer)
            BS_TRY(launch_resid_sum(w.x, w.part_o, w.ks_o, (size_t)M * d, L.ffn_norm, d, M, fuse_gu ? (size_t)16 * d : (size_t)M * d, w.h, w.ssq,
                                    fuse_gu, s));
        else
            BS_TRY(launch_rmsnorm(dt, w.x, w.part_o, w.ks_o, (size_t)M * d, L.ffn_norm, d, c.norm_eps, B, q_len, q_len,
                                  (size_t)M * d, w.h, s));
        }
        g.x = w.h; g.x_plane = (size_t)M * d; g.w[0] = L.w_gate; g.w[1] = L.w_up; g.w[2] = nullptr; g.seg_rows[0] = ff; g.seg_rows[1] = ff;
        g.out = w.part_gu; g.ks_stride = (size_t)M * 2 * ff; g.M = M; g.N = 2 * ff; g.K = d; g.ldo = 2 * ff; g.KS = w.ks_gu;
        if (fuse_gu) {
            DecArgs a = {};
            a.xh = reinterpret_cast<const uint16_t*>(w.h); a.x_plane = (size_t)16 * d; a.w[0] = L.w_gate; a.w[1] = L.w_up;
            a.M = M; a.N = ff; a.K = d; a.ssq_in = w.ssq; a.ssq_tiles = fuse_o ? d / 16 : ssq_chunks; a.eps = c.norm_eps;
            a.out_planes = reinterpret_cast<uint16_t*>(w.act); a.out_plane = fuse_d ? (size_t)16 * ff : (size_t)M * ff; a.out_tiled = fuse_d ? 1 : 0;
            BS_TRY(launch_gemm_rows(EPI_SWIGLU, a, s));
        } else {
        BS_TRY(launch_gemm(dt, g, s));
        BS_TRY(launch_swiglu(dt, w.part_gu, w.ks_gu, (size_t)M * 2 * ff, M, ff, (size_t)M * ff, w.act, ssq, d, c.norm_eps, s));
        }
        g.x = w.act; g.x_plane = (size_t)M * ff; g.w[0] = L.w_down; g.w[1] = g.w[2] = nullptr; g.seg_rows[0] = d; g.seg_rows[1] = 0;
        g.out = w.part_d; g.ks_stride = (size_t)M * d; g.M = M; g.N = d; g.K = ff; g.ldo = d; g.KS = w.ks_d;
        if (fuse_d) {
            const bool more = l + 1 < c.n_layers;
            DecArgs a = {};
            a.xh = reinterpret_cast<const uint16_t*>(w.act); a.x_plane = (size_t)16 * ff; a.w[0] = L.w_down; a.M = M; a.N = d; a.K = ff;
            a.x = w.x; a.gain_next = more ? m->layers[l + 1].attn_norm : nullptr;
            a.out_planes = reinterpret_cast<uint16_t*>(w.h); a.out_plane = (size_t)16 * d; a.out_tiled = 1;
            a.ssq_out = more ? w.ssq : nullptr;
            BS_TRY(launch_gemm_rows(EPI_RESID, a, s));
        } else {
        BS_TRY(launch_gemm(dt, g, s));
        pend = w.part_d;
        }
    }
    }
    if (logit_rows > 0) {
        const int R = B * logit_rows;
        BS_TRY(launch_rmsnorm(dt, w.x, pend, w.ks_d, (size_t)M * d, m->final_norm, d, c.norm_eps, B, q_len, logit_rows,
                              (size_t)R * d, w.h, s));
        GemmArgs g;
        g.tiled = m->packed ? 1 : 0;
        g.x_plane = (size_t)R * d;
        g.w[0] = m->lm_head; g.w[1] = g.w[2] = nullptr; g.seg_rows[0] = c.vocab; g.seg_rows[1] = 0;
        g.N = c.vocab; g.K = d; g.KS = 1; g.ks_stride = 0;
        if (logits_bstride == (size_t)logit_rows * c.vocab) {            // rows of all sequences contiguous
            g.x = w.h; g.out = logits; g.M = R; g.ldo = c.vocab;
            BS_TRY(launch_gemm(dt, g, s));
        } else if (logit_rows == 1) {                                     // one row per sequence, strided output
            g.x = w.h; g.out = logits; g.M = B; g.ldo = (int)logits_bstride;
            BS_TRY(launch_gemm(dt, g, s));
        } else {
            for (int b = 0; b < B; ++b) {
                g.x = reinterpret_cast<char*>(w.h) + (size_t)b * logit_rows * d * (dt == BS_BF16 ? 2 : 4);
                g.out = logits + (size_t)b * logits_bstride; g.M = logit_rows; g.ldo = c.vocab;
                BS_TRY(launch_gemm(dt, g, s));
            }
        }
    }
#undef BS_TRY
    return BS_OK;
}

static int check_fwd_args(const bs_model* m, const bs_kv* kv, const char* who) {
    BS_REQUIRE(m && kv, BS_EINVAL, "%s: NULL handle", who);
    const bs_model_cfg &a = m->cfg, &b = kv->cfg;
    BS_REQUIRE(a.n_layers == b.n_layers && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim && a.dtype == b.dtype,
               BS_ESTATE, "%s: KV cache was bound for a different model shape", who);
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_verify_forward(const bs_model* m, const bs_kv* kv, const int32_t* dev_q_tokens, const int32_t* dev_kv_len,
                                 int q_len, int logit_rows, float* dev_logits, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_fwd_args(m, kv, "bs_verify_forward");
    if (rc != BS_OK) return rc;
    BS_REQUIRE(dev_q_tokens && dev_kv_len && ws, BS_EINVAL, "bs_verify_forward: NULL pointer");
    BS_REQUIRE(q_len >= 1 && q_len <= kv->max_len, BS_ESHAPE, "bs_verify_forward: q_len=%d outside [1, max_len=%d]", q_len, kv->max_len);
    BS_REQUIRE(logit_rows >= 0 && logit_rows <= q_len, BS_ESHAPE, "bs_verify_forward: logit_rows=%d outside [0, q_len=%d]", logit_rows, q_len);
    BS_REQUIRE(logit_rows == 0 || dev_logits, BS_EINVAL, "bs_verify_forward: dev_logits is NULL");
    BS_REQUIRE((long long)kv->B * q_len <= (1 << 20), BS_ESHAPE, "bs_verify_forward: too many query rows");
    return forward(m, kv, dev_q_tokens, q_len, dev_kv_len, 0, q_len, logit_rows, dev_logits, (size_t)logit_rows * m->cfg.vocab,
                   ws, ws_bytes, reinterpret_cast<hipStream_t>(stream));
}

extern "C" __attribute__((visibility("default"))) int bs_prefill(const bs_model* m, const bs_kv* kv, const int32_t* dev_tokens, int token_stride, int n,
                          float* dev_last_logits, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_fwd_args(m, kv, "bs_prefill");
    if (rc != BS_OK) return rc;
    BS_REQUIRE(dev_tokens && ws, BS_EINVAL, "bs_prefill: NULL pointer");
    BS_REQUIRE(n >= 1 && n <= token_stride && n <= kv->max_len, BS_ESHAPE, "bs_prefill: n=%d, stride=%d, max_len=%d", n, token_stride, kv->max_len);
    // largest chunk the workspace allows: at most 128 query rows per sequence, 1024 for a single sequence (blocks of
    // 256 rows share a GEMM launch: more rows mean more workgroups per weight tile, fewer splits of K, and so fewer
    // partial sums written and re-read per multiply)
    const int cap = kv->B == 1 ? 1024 : 128;
    int chunk = n < cap ? n : cap;
    while (chunk > 1 && bs_forward_workspace_bytes(&m->cfg, kv->B, chunk, kv->max_len) > ws_bytes) chunk /= 2;
    BS_REQUIRE(bs_forward_workspace_bytes(&m->cfg, kv->B, chunk, kv->max_len) <= ws_bytes, BS_EWORKSPACE,
               "bs_prefill: workspace %zu bytes too small even for one row per sequence", ws_bytes);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    for (int start = 0; start < n; start += chunk) {
        const int len = (n - start < chunk) ? n - start : chunk;
        const bool last = start + len >= n;
        rc = forward(m, kv, dev_tokens + start, token_stride, nullptr, start, len, (last && dev_last_logits) ? 1 : 0,
                     dev_last_logits, (size_t)m->cfg.vocab, ws, ws_bytes, s);
        if (rc != BS_OK) return rc;
    }
    return BS_OK;
}

// =====================================================================================================
// Round driver
// =====================================================================================================
struct RoundWs {
    uint32_t* round; int32_t* status;
    int32_t *q_draft2, *q_draft1, *q_target, *draft_tokens, *kvlen_draft, *kvlen_target, *flags, *cand, *active;
    float *draft_logits, *target_logits, *margins; void* stats;
    float* sigma;            // [B] draft-logit noise scale of this round
    int32_t* dlen;           // [n_drafts][B] tokens whose keys/values each draft cache holds
    int32_t *q_catch, *kvlen_catch;     // inputs of a catch-up pass
    char* fwd; size_t fwd_bytes; size_t total;
};

constexpr int CATCH = 16;    // tokens per sequence one catch-up pass of an idle draft model processes

static RoundWs carve_round(const bs_model_cfg& t, const bs_model_cfg* const* drafts, int n_drafts, int B, int L, int max_len, char* base) {
    RoundWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return base ? base + o : (char*)nullptr; };
    char* hdr = take(256);
    w.round = (uint32_t*)hdr; w.status = (int32_t*)(hdr ? hdr + 64 : nullptr);
    w.q_draft2 = (int32_t*)take((size_t)B * 2 * 4);
    w.q_draft1 = (int32_t*)take((size_t)B * 4);
    w.q_target = (int32_t*)take((size_t)B * (L + 1) * 4);
    w.draft_tokens = (int32_t*)take((size_t)B * L * 4);
    w.kvlen_draft = (int32_t*)take((size_t)B * 4);
    w.kvlen_target = (int32_t*)take((size_t)B * 4);
    w.flags = (int32_t*)take((size_t)B * (L + 1) * 4);
    w.cand = (int32_t*)take((size_t)B * (L + 1) * 4);
    w.active = (int32_t*)take((size_t)B * 4);
    w.margins = (float*)take((size_t)B * L * 4);
    w.stats = take(spec_scratch_bytes(B, L));
    w.sigma = (float*)take((size_t)B * 4);
    w.dlen = (int32_t*)take((size_t)n_drafts * B * 4);
    w.q_catch = (int32_t*)take((size_t)B * CATCH * 4);
    w.kvlen_catch = (int32_t*)take((size_t)B * 4);
    w.draft_logits = (float*)take((size_t)B * L * t.vocab * 4);
    w.target_logits = (float*)take((size_t)B * (L + 1) * t.vocab * 4);
    size_t f = carve_max(t, B, L + 1, max_len);
    for (int i = 0; i < n_drafts; ++i) {
        size_t fd = carve_max(*drafts[i], B, max_len >= CATCH ? CATCH : 2, max_len);      // draft steps (1-2 rows) and catch-up passes
        if (fd > f) f = fd;
    }
    w.fwd = take(f); w.fwd_bytes = f;
    w.total = off;
    return w;
}

extern "C" __attribute__((visibility("default"))) size_t bs_round_workspace_bytes(const bs_model_cfg* target, const bs_model_cfg* const* drafts, int n_drafts,
                                                   int B, int L, int max_len) {
    if (!target || !drafts || n_drafts < 1 || B < 1 || L < 0 || max_len < 1) return 0;
    return carve_round(*target, drafts, n_drafts, B, L, max_len, nullptr).total;
}

struct ArmGraph {
    hipGraphExec_t exec = nullptr;
    int32_t* emitted = nullptr; int32_t* n_emitted = nullptr; hipStream_t stream = nullptr;
};

struct bs_round {
    bs_round_cfg cfg;
    std::vector<const bs_model*> drafts;
    std::vector<const bs_kv*> draft_kvs;
    std::vector<int> arm_draft, arm_gamma;
    int L;
    RoundWs ws;
    std::vector<ArmGraph> graphs;
    std::vector<int> lag_bound;      // per draft: upper bound of the tokens emitted since its cache was last brought up to date
    int last_gamma;
};

namespace bs {

__global__ void set_round_kernel(uint32_t* round, int32_t* status, int32_t* fwd_status, uint32_t t0,
                                 const int32_t* __restrict__ total_len, int B, int n_drafts, int32_t* __restrict__ dlen) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { *round = t0; *status = 0; *fwd_status = 0; }
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * n_drafts) dlen[i] = total_len[i % B];       // caller's promise: caches are filled for the current tokens
}

// Inputs of one catch-up pass of a draft model whose cache lags: CATCH tokens per sequence from the first position
// the cache does not hold yet (never past total-2: the round's first draft step feeds the last two tokens itself).
__global__ void catchup_prepare_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ total_len, int B,
                                       int max_len, int32_t* __restrict__ dlen, int32_t* __restrict__ q_catch,
                                       int32_t* __restrict__ kvlen_catch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int total = total_len[b];
    if (total < 2 || total > max_len) { kvlen_catch[b] = max_len; return; }       // the forward skips this sequence
    const int need = total - 2;
    const int have = min(dlen[b], need);
    const int start = max(min(have, max_len - CATCH), 0);                          // the pass must fit the cache
    for (int j = 0; j < CATCH; ++j) {
        const int pos = start + j;
        q_catch[b * CATCH + j] = pos < total ? tokens[(size_t)b * max_len + pos] : 0;   // past the end: rows nobody reads
    }
    kvlen_catch[b] = start;
    dlen[b] = max(have, min(start + CATCH, need));
}

// Draft-logit perturbation: row[v] += sigma[b] * z(b, t, i, v) with Box-Muller normals from Philox
// (counter (b, t, i, 4 + 8g) -> four words for v = 4g..4g+3).  grid (ceil(V/4/256), B).
__global__ void noise_kernel(float* __restrict__ rows, size_t row_stride, int V, const float* __restrict__ sigma,
                             uint64_t seed, const uint32_t* __restrict__ round, uint32_t slot) {
    const int b = blockIdx.y;
    const float sg = sigma[b];
    if (sg == 0.f) return;
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (4 * g >= V) return;
    const Philox4 ph = philox4(seed, (uint32_t)b, *round, slot, PURPOSE_NOISE + 8u * (uint32_t)g);
    float z[4];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        const float u1 = u_open_closed(ph.w[2 * pr]), u2 = u_closed_open(ph.w[2 * pr + 1]);
        const float rad = sqrtf(-2.0f * logf(u1));
        float sn, cs;
        sincosf(6.28318530717958647692f * u2, &sn, &cs);
        z[2 * pr] = rad * cs; z[2 * pr + 1] = rad * sn;
    }
    float* row = rows + (size_t)b * row_stride;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (4 * g + e < V) row[4 * g + e] += sg * z[e];
}

// Start of a round: gather the draft's first two inputs and the target's first query token.  A sequence takes part
// only if the whole round fits its caches: the verification pass writes keys at total-1 .. total-1+gamma and the draft
// steps stay below that, so total + gamma <= max_len.  One that does not fit is skipped by every forward pass of the
// round (cache length max_len), emits nothing and commits nothing; status bit 8 says so if it was still generating.
__global__ void round_begin_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ total_len,
                                   const int32_t* __restrict__ goal_len, int B, int max_len, int gamma, int tq_stride,
                                   int32_t* __restrict__ q_draft2, int32_t* __restrict__ q_target,
                                   int32_t* __restrict__ kvlen_draft, int32_t* __restrict__ kvlen_target,
                                   int32_t* __restrict__ active, int32_t* __restrict__ status,
                                   const int32_t* __restrict__ prompt_len, float sigma_a, float sigma_b, int period,
                                   float* __restrict__ sigma) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int total = total_len[b];
    {
        const int generated = max(total - (prompt_len ? prompt_len[b] : 0), 0);
        sigma[b] = (period > 0 && ((generated / period) & 1)) ? sigma_b : sigma_a;
    }
    const bool sane = total >= 2 && total <= max_len;
    const bool ok = sane && total + gamma <= max_len;
    const bool wants = goal_len == nullptr || total < goal_len[b];
    if (!sane) atomicOr(status, 4);
    else if (!ok && wants) atomicOr(status, 8);
    const int t1 = ok ? tokens[(size_t)b * max_len + total - 1] : 0;
    const int t0 = ok ? tokens[(size_t)b * max_len + total - 2] : 0;
    q_draft2[2 * b] = t0; q_draft2[2 * b + 1] = t1;
    q_target[(size_t)b * tq_stride] = t1;
    kvlen_draft[b] = ok ? total - 2 : max_len;        // max_len: makes the forward skip the sequence
    kvlen_target[b] = ok ? total - 1 : max_len;
    active[b] = ok && wants;
}

// End of a round (Alg. 3: pt_t = concat(pt_{t-1}, x_t); reward y = len(x_t)).
__global__ void round_commit_kernel(const int32_t* __restrict__ flags, const int32_t* __restrict__ cand,
                                    const int32_t* __restrict__ draft_tokens, const int32_t* __restrict__ active,
                                    const int32_t* __restrict__ goal_len, int B, int gamma, int L, int max_len,
                                    int32_t* __restrict__ tokens, int32_t* __restrict__ total_len,
                                    int32_t* __restrict__ emitted, int32_t* __restrict__ n_emitted,
                                    uint32_t* __restrict__ round, int32_t* __restrict__ dlen_used) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b == 0) *round += 1u;      // every kernel of this round has already read the counter (stream order)
    if (b >= B) return;
    if (!active[b]) { n_emitted[b] = 0; return; }
    int tau = 0;
    while (tau < gamma && (flags[(size_t)b * (gamma + 1) + tau] & 1)) ++tau;
    const int total = total_len[b];
    // the draft's steps consumed x~_1 .. x~_{gamma-1}: its cache is right up to the last accepted one of those
    if (dlen_used) dlen_used[b] = total + min(tau, gamma - 1);
    const int goal = goal_len ? min(goal_len[b], max_len) : max_len;
    int len = total;
    for (int i = 0; i <= tau; ++i) {
        const int tk = (i < tau) ? draft_tokens[(size_t)b * gamma + i] : cand[(size_t)b * (gamma + 1) + tau];
        emitted[(size_t)b * (L + 1) + i] = tk;
        if (len < goal) { tokens[(size_t)b * max_len + len] = tk; ++len; }
    }
    for (int i = tau + 1; i <= L; ++i) emitted[(size_t)b * (L + 1) + i] = -1;
    total_len[b] = len;
    n_emitted[b] = tau + 1;
}

}  // namespace bs

extern "C" __attribute__((visibility("default"))) int bs_round_create(const bs_round_cfg* cfg, bs_round** out) {
    BS_REQUIRE(cfg && out, BS_EINVAL, "bs_round_create: NULL argument");
    BS_REQUIRE(cfg->target && cfg->target_kv && cfg->drafts && cfg->draft_kvs && cfg->arm_draft && cfg->arm_gamma, BS_EINVAL,
               "bs_round_create: NULL handle array");
    BS_REQUIRE(cfg->dev_tokens && cfg->dev_total_len && cfg->dev_workspace, BS_EINVAL, "bs_round_create: NULL device pointer");
    BS_REQUIRE(cfg->n_drafts >= 1 && cfg->n_arms >= 1 && cfg->B >= 1 && cfg->max_len >= 2, BS_ESHAPE, "bs_round_create: bad counts");
    BS_REQUIRE(cfg->temperature >= 0.f, BS_EINVAL, "bs_round_create: temperature must be >= 0");
    BS_REQUIRE(cfg->noise_sigma[0] >= 0.f && cfg->noise_sigma[1] >= 0.f && cfg->noise_period >= 0, BS_EINVAL,
               "bs_round_create: noise scale and period must be >= 0");
    {
        bool idle_possible = cfg->n_drafts > 1;                   // a draft model can miss rounds: other drafts, or gamma = 0 arms
        for (int a = 0; a < cfg->n_arms; ++a) idle_possible = idle_possible || cfg->arm_gamma[a] == 0;
        BS_REQUIRE(!idle_possible || cfg->max_len >= CATCH, BS_ESHAPE,
                   "bs_round_create: several draft models or gamma = 0 arms need max_len >= %d", CATCH);
    }
    int rc = check_fwd_args(cfg->target, cfg->target_kv, "bs_round_create(target)");
    if (rc != BS_OK) return rc;
    BS_REQUIRE(cfg->target_kv->B == cfg->B && cfg->target_kv->max_len == cfg->max_len, BS_ESHAPE,
               "bs_round_create: target cache bound for B=%d max_len=%d", cfg->target_kv->B, cfg->target_kv->max_len);
    std::vector<const bs_model_cfg*> dcfg;
    for (int i = 0; i < cfg->n_drafts; ++i) {
        rc = check_fwd_args(cfg->drafts[i], cfg->draft_kvs[i], "bs_round_create(draft)");
        if (rc != BS_OK) return rc;
        BS_REQUIRE(cfg->draft_kvs[i]->B == cfg->B && cfg->draft_kvs[i]->max_len == cfg->max_len, BS_ESHAPE,
                   "bs_round_create: draft %d cache bound for another B/max_len", i);
        BS_REQUIRE(cfg->drafts[i]->cfg.vocab == cfg->target->cfg.vocab, BS_ESHAPE, "bs_round_create: draft %d vocabulary differs", i);
        dcfg.push_back(&cfg->drafts[i]->cfg);
    }
    int L = 0;
    for (int a = 0; a < cfg->n_arms; ++a) {
        BS_REQUIRE(cfg->arm_draft[a] >= 0 && cfg->arm_draft[a] < cfg->n_drafts, BS_EINVAL, "bs_round_create: arm %d names draft %d", a, cfg->arm_draft[a]);
        BS_REQUIRE(cfg->arm_gamma[a] >= 0 && cfg->arm_gamma[a] <= 64, BS_EINVAL, "bs_round_create: arm %d gamma %d outside [0,64]", a, cfg->arm_gamma[a]);
        if (cfg->arm_gamma[a] > L) L = cfg->arm_gamma[a];
    }
    const size_t need = carve_round(cfg->target->cfg, dcfg.data(), cfg->n_drafts, cfg->B, L, cfg->max_len, nullptr).total;
    BS_REQUIRE(cfg->workspace_bytes >= need, BS_EWORKSPACE, "bs_round_create: workspace %zu < %zu bytes", cfg->workspace_bytes, need);
    BS_REQUIRE((reinterpret_cast<uintptr_t>(cfg->dev_workspace) & 255) == 0, BS_EWORKSPACE, "bs_round_create: workspace not 256-byte aligned");
    bs_round* r = new (std::nothrow) bs_round();
    BS_REQUIRE(r, BS_EINVAL, "bs_round_create: out of host memory");
    r->cfg = *cfg;
    r->drafts.assign(cfg->drafts, cfg->drafts + cfg->n_drafts);
    r->draft_kvs.assign(cfg->draft_kvs, cfg->draft_kvs + cfg->n_drafts);
    r->arm_draft.assign(cfg->arm_draft, cfg->arm_draft + cfg->n_arms);
    r->arm_gamma.assign(cfg->arm_gamma, cfg->arm_gamma + cfg->n_arms);
    r->L = L;
    r->ws = carve_round(cfg->target->cfg, dcfg.data(), cfg->n_drafts, cfg->B, L, cfg->max_len, reinterpret_cast<char*>(cfg->dev_workspace));
    r->graphs.resize(cfg->n_arms);
    r->lag_bound.assign(cfg->n_drafts, 0);
    r->last_gamma = 0;
    *out = r;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_round_destroy(bs_round* r) {
    if (r) {
        for (auto& g : r->graphs)
            if (g.exec) (void)hipGraphExecDestroy(g.exec);
        delete r;
    }
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_round_reset(bs_round* r, uint32_t t0, void* stream) {
    BS_REQUIRE(r, BS_EINVAL, "bs_round_reset: NULL handle");
    const int n = r->cfg.B * r->cfg.n_drafts;
    hipLaunchKernelGGL(bs::set_round_kernel, dim3((n + 127) / 128), dim3(128), 0, reinterpret_cast<hipStream_t>(stream), r->ws.round,
                       r->ws.status, reinterpret_cast<int32_t*>(r->ws.fwd), t0, r->cfg.dev_total_len, r->cfg.B, r->cfg.n_drafts, r->ws.dlen);
    BS_LAUNCH_CHECK();
    r->lag_bound.assign(r->cfg.n_drafts, 0);
    return BS_OK;
}

// Brings the cache of the arm's draft model up to total_len-2 if it was idle (eager launches, outside any graph).
static int catch_up(bs_round* r, int arm, hipStream_t s) {
    const bs_round_cfg& c = r->cfg;
    const int d = r->arm_draft[arm], B = c.B;
    RoundWs& w = r->ws;
    const int passes = (r->lag_bound[d] + CATCH - 1) / CATCH;
    for (int p = 0; p < passes; ++p) {
        hipLaunchKernelGGL(bs::catchup_prepare_kernel, dim3((B + 127) / 128), dim3(128), 0, s, c.dev_tokens, c.dev_total_len, B,
                           c.max_len, w.dlen + (size_t)d * B, w.q_catch, w.kvlen_catch);
        BS_LAUNCH_CHECK();
        const int rc = forward(r->drafts[d], r->draft_kvs[d], w.q_catch, CATCH, w.kvlen_catch, 0, CATCH, 0, nullptr, 0, w.fwd, w.fwd_bytes, s);
        if (rc != BS_OK) return rc;
    }
    r->lag_bound[d] = 0;
    return BS_OK;
}

// round_begin + the gamma draft steps of the arm (App. A, generation of x~_1..x~_gamma)
static int enqueue_draft(bs_round* r, int arm, hipStream_t s) {
    const bs_round_cfg& c = r->cfg;
    const int gamma = r->arm_gamma[arm], B = c.B, V = c.target->cfg.vocab;
    const bs_model* draft = r->drafts[r->arm_draft[arm]];
    const bs_kv* dkv = r->draft_kvs[r->arm_draft[arm]];
    RoundWs& w = r->ws;
    const bool noisy = c.noise_sigma[0] > 0.f || c.noise_sigma[1] > 0.f;
    int rc;
    hipLaunchKernelGGL(bs::round_begin_kernel, dim3((B + 127) / 128), dim3(128), 0, s, c.dev_tokens, c.dev_total_len,
                       c.dev_goal_len, B, c.max_len, gamma, gamma + 1, w.q_draft2, w.q_target, w.kvlen_draft, w.kvlen_target,
                       w.active, w.status, c.dev_prompt_len, c.noise_sigma[0], c.noise_sigma[1], c.noise_period, w.sigma);
    BS_LAUNCH_CHECK();
    for (int i = 0; i < gamma; ++i) {
        float* row = w.draft_logits + (size_t)i * V;                  // [B, gamma, V], row i of every sequence
        if (i == 0)
            rc = forward(draft, dkv, w.q_draft2, 2, w.kvlen_draft, 0, 2, 1, row, (size_t)gamma * V, w.fwd, w.fwd_bytes, s);
        else
            rc = forward(draft, dkv, w.q_draft1, 1, w.kvlen_draft, i + 1, 1, 1, row, (size_t)gamma * V, w.fwd, w.fwd_bytes, s);
        if (rc != BS_OK) return rc;
        if (noisy) {
            hipLaunchKernelGGL(bs::noise_kernel, dim3(((V + 3) / 4 + 255) / 256, B), dim3(256), 0, s, row, (size_t)gamma * V, V,
                               w.sigma, c.seed, w.round, (uint32_t)i);
            BS_LAUNCH_CHECK();
        }
        DrawParams d;
        d.logits = row; d.row_stride = gamma * V; d.V = V; d.seed = c.seed;
        d.greedy = c.temperature == 0.f ? 1 : 0;
        d.inv_temp = d.greedy ? 1.0f : 1.0f / c.temperature;
        d.round_ptr = w.round; d.round = 0; d.slot = (uint32_t)i;
        d.out0 = w.draft_tokens; d.stride0 = gamma; d.off0 = i;
        d.out1 = w.q_target; d.stride1 = gamma + 1; d.off1 = i + 1;
        d.out2 = w.q_draft1; d.stride2 = 1; d.off2 = 0;
        rc = launch_draw(d, B, s);
        if (rc != BS_OK) return rc;
    }
    return BS_OK;
}

static int enqueue_round(bs_round* r, int arm, int32_t* emitted, int32_t* n_emitted, hipStream_t s) {
    const bs_round_cfg& c = r->cfg;
    const int gamma = r->arm_gamma[arm], B = c.B, V = c.target->cfg.vocab;
    RoundWs& w = r->ws;
    int rc = enqueue_draft(r, arm, s);
    if (rc != BS_OK) return rc;
    // ---- verification: one target pass over gamma+1 positions ----
    rc = forward(c.target, c.target_kv, w.q_target, gamma + 1, w.kvlen_target, 0, gamma + 1, gamma + 1, w.target_logits,
                 (size_t)(gamma + 1) * V, w.fwd, w.fwd_bytes, s);
    if (rc != BS_OK) return rc;
    // ---- accept / reject, residual and bonus candidates ----
    rc = launch_spec_sample(w.target_logits, w.draft_logits, w.draft_tokens, B, gamma, V, BS_F32, c.temperature, nullptr,
                            c.seed, w.round, 0, w.stats, w.flags, w.cand, nullptr, nullptr, w.margins, s);
    if (rc != BS_OK) return rc;
    // ---- commit ----
    hipLaunchKernelGGL(bs::round_commit_kernel, dim3((B + 127) / 128), dim3(128), 0, s, w.flags, w.cand, w.draft_tokens,
                       w.active, c.dev_goal_len, B, gamma, r->L, c.max_len, c.dev_tokens, c.dev_total_len, emitted,
                       n_emitted, w.round, gamma > 0 ? w.dlen + (size_t)r->arm_draft[arm] * B : nullptr);
    BS_LAUNCH_CHECK();
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_spec_round(bs_round* r, int arm, int32_t* dev_emitted, int32_t* dev_n_emitted, void* stream) {
    BS_REQUIRE(r, BS_EINVAL, "bs_spec_round: NULL handle");
    BS_REQUIRE(arm >= 0 && arm < (int)r->arm_gamma.size(), BS_EINVAL, "bs_spec_round: arm %d not in [0,%zu)", arm, r->arm_gamma.size());
    BS_REQUIRE(dev_emitted && dev_n_emitted, BS_EINVAL, "bs_spec_round: NULL output pointer");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    r->last_gamma = r->arm_gamma[arm];
    {
        const bool drafts_used = r->arm_gamma[arm] > 0;
        if (drafts_used) {
            const int rc = catch_up(r, arm, s);
            if (rc != BS_OK) return rc;
        }
        for (size_t d = 0; d < r->lag_bound.size(); ++d)          // the drafts not used fall behind by what this round emits
            if (!drafts_used || (int)d != r->arm_draft[arm]) r->lag_bound[d] += r->arm_gamma[arm] + 1;
    }
    if (!r->cfg.use_graph) return enqueue_round(r, arm, dev_emitted, dev_n_emitted, s);
    BS_REQUIRE(s != nullptr, BS_EINVAL, "bs_spec_round: graph mode needs a non-null stream");
    ArmGraph& g = r->graphs[arm];
    if (g.exec && (g.emitted != dev_emitted || g.n_emitted != dev_n_emitted)) {
        (void)hipGraphExecDestroy(g.exec);
        g.exec = nullptr;
    }
    if (!g.exec) {
        hipGraph_t graph = nullptr;
        BS_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
        const int rc = enqueue_round(r, arm, dev_emitted, dev_n_emitted, s);
        const hipError_t e = hipStreamEndCapture(s, &graph);
        if (rc != BS_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e != hipSuccess) BS_FAIL(BS_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
        const hipError_t e2 = hipGraphInstantiate(&g.exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e2 != hipSuccess) { g.exec = nullptr; BS_FAIL(BS_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e2)); }
        g.emitted = dev_emitted; g.n_emitted = dev_n_emitted;
    }
    BS_HIP(hipGraphLaunch(g.exec, s));
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_draft_propose(bs_round* r, int arm, int32_t* dev_draft_tokens, float* dev_draft_logits, void* stream) {
    BS_REQUIRE(r, BS_EINVAL, "bs_draft_propose: NULL handle");
    BS_REQUIRE(arm >= 0 && arm < (int)r->arm_gamma.size(), BS_EINVAL, "bs_draft_propose: arm %d not in [0,%zu)", arm, r->arm_gamma.size());
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    int rc = catch_up(r, arm, s);
    if (rc != BS_OK) return rc;
    rc = enqueue_draft(r, arm, s);
    if (rc != BS_OK) return rc;
    const int gamma = r->arm_gamma[arm], B = r->cfg.B, V = r->cfg.target->cfg.vocab;
    if (dev_draft_tokens) BS_HIP(hipMemcpyAsync(dev_draft_tokens, r->ws.draft_tokens, (size_t)B * gamma * 4, hipMemcpyDeviceToDevice, s));
    if (dev_draft_logits) BS_HIP(hipMemcpyAsync(dev_draft_logits, r->ws.draft_logits, (size_t)B * gamma * V * 4, hipMemcpyDeviceToDevice, s));
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_round_status(bs_round* r, int32_t* host_out, void* stream) {
    BS_REQUIRE(r && host_out, BS_EINVAL, "bs_round_status: NULL argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    int32_t words[2] = {0, 0};
    BS_HIP(hipMemcpyAsync(&words[0], r->ws.status, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    BS_HIP(hipMemcpyAsync(&words[1], r->ws.fwd, sizeof(int32_t), hipMemcpyDeviceToHost, s));      // the forward passes' word
    BS_HIP(hipStreamSynchronize(s));
    *host_out = words[0] | words[1];
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_round_debug_views(bs_round* r, const float** tl, const float** dl, const int32_t** dt, const float** mg) {
    BS_REQUIRE(r, BS_EINVAL, "bs_round_debug_views: NULL handle");
    if (tl) *tl = r->ws.target_logits;
    if (dl) *dl = r->ws.draft_logits;
    if (dt) *dt = r->ws.draft_tokens;
    if (mg) *mg = r->ws.margins;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_step_poll_limit(unsigned polls) {
    g_step_polls.store(polls ? polls : STEP_DEFAULT_POLLS);
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_profile_enable(int on) { return bs::profile_enable(on); }
extern "C" __attribute__((visibility("default"))) int bs_profile_collect(int row_tiles, double* total_ms, double* total_bytes, long long* launches) {
    return bs::profile_collect(row_tiles, total_ms, total_bytes, launches);
}
