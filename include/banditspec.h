/*
 * banditspec.h - C ABI of the MI355X (gfx950) hot path of BanditSpec (arXiv 2505.15141).
 *
 * One speculative-decoding round = the subroutine of Alg. 2 instantiated with vanilla speculative
 * decoding (App. A): gamma draft draws, one target pass over gamma+1 query positions, accept/reject
 * with residual / bonus sampling.  The arm-selection rules UCBSpec (Alg. 4) and EXP3Spec (Alg. 5)
 * run on the host between rounds (Alg. 3).
 *
 * Conventions
 *  - Every function returns an int status: BS_OK (0) or a negative bs_status.  bs_last_error_string()
 *    gives the detail for the calling thread.  Nothing throws, nothing aborts.
 *  - Pointers named dev_* are DEVICE pointers, host_* / plain structs are HOST memory.  All device
 *    memory (weights, KV caches, tokens, logits, workspaces) is owned by the caller and must stay
 *    alive until the stream work of the call has finished.  The library allocates no device memory.
 *    It owns only the small host handles it creates (create/destroy pairs).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only enqueue work;
 *    they never synchronise unless stated.
 *  - Matrices are row-major [out_features, in_features] (y = x W^T), in the model dtype.
 *    Norm gains are float32.  Logits are always float32 on the model path.
 *  - Shapes and arguments are validated on the host before anything is launched.
 */
#ifndef BANDITSPEC_H
#define BANDITSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BS_OK = 0,
    BS_EINVAL = -1,     /* null pointer, value out of range */
    BS_ESHAPE = -2,     /* sizes that do not fit together or exceed a kernel limit */
    BS_EDTYPE = -3,     /* unknown or unsupported dtype */
    BS_EWORKSPACE = -4, /* workspace too small or misaligned */
    BS_ESTATE = -5,     /* call order / handle state */
    BS_EHIP = -6        /* a HIP runtime call failed */
} bs_status;

typedef enum { BS_F32 = 0, BS_BF16 = 1 } bs_dtype;

const char* bs_last_error_string(void);
int bs_version(void);

/* ------------------------------------------------------------------------------------------------
 * Philox4x32-10 word used by every random decision (host function, for parity checks).
 * Counter = (b, t, slot, purpose), key = seed.  purpose: 0 draft draw, 1 acceptance test,
 * 2 residual/bonus draw, 3 EXP3Spec arm draw.  Acceptance uniforms are ((w>>8)+1)*2^-24 in (0,1],
 * draw uniforms (w>>8)*2^-24 in [0,1).
 * ---------------------------------------------------------------------------------------------- */
uint32_t bs_philox_word(uint64_t seed, uint32_t b, uint32_t t, uint32_t slot, uint32_t purpose);

/* ------------------------------------------------------------------------------------------------
 * Accept/reject + residual/bonus sampling (App. A, vanilla speculative decoding, the loop over draft
 * positions and the bonus draw).  For each sequence b:
 *   tau = number of leading draft positions i with  u_i <= min{1, p_i(x~_i) / q_i(x~_i)}  (tested as
 *         u_i * q_i(x~_i) <= p_i(x~_i)),  p_i = softmax(target_logits[b,i]/T), q_i likewise;
 *   next_token ~ Norm([p_{tau+1} - q_{tau+1}]_+) if tau < gamma, else ~ p_{gamma+1};
 *   draws are inverse-CDF in increasing token id with one uniform in [0,1).
 *
 *  dev_target_logits [B, gamma+1, V], dev_draft_logits [B, gamma, V]  contiguous, `dtype` elements
 *  dev_draft_tokens  [B, gamma] int32, each in [0, V)
 *  dev_uniforms      [B, gamma+1] float32 (columns 0..gamma-1 acceptance, column gamma final draw),
 *                    or NULL: then Philox(seed; b, round, i, purpose) is generated in the kernel
 *  dev_accept_len    [B] int32 out (tau);  dev_next_token [B] int32 out
 *  dev_margins       [B, gamma] float32 out or NULL: min(1,p/q) - u for every position (all tested)
 *  dev_workspace     bs_spec_sample_workspace_bytes(B, gamma) bytes, 16-byte aligned, contents ignored
 *                    (per-row softmax statistics)
 * 0 <= gamma <= 512, B >= 0 (B == 0 is a no-op), 1 <= V <= 2^20, temperature >= 0.
 * temperature == 0 is greedy decoding, the limit T -> 0 of Sec. 2: p_i and q_i put all mass on their largest logit
 * (lowest token id among equal ones), so a draft token is accepted iff it is the target's argmax at its position and
 * next_token is the target's argmax at the deciding position; no uniform is used, dev_draft_logits may be NULL (the
 * draft tokens are taken to be the draft's argmax), margins are +1 / -1.
 * ---------------------------------------------------------------------------------------------- */
size_t bs_spec_sample_workspace_bytes(int B, int gamma);
int bs_spec_sample(const void* dev_target_logits, const void* dev_draft_logits,
                   const int32_t* dev_draft_tokens, int B, int gamma, int V, int dtype,
                   float temperature, const float* dev_uniforms, uint64_t seed, uint32_t round,
                   int32_t* dev_accept_len, int32_t* dev_next_token, float* dev_margins,
                   void* dev_workspace, size_t workspace_bytes, void* stream);

/* The same operation for callers that cannot allocate device memory or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the per-row statistics go to a static array in device memory
 * that every GPU the library runs on holds until the process ends (512 KiB).  Same arguments and results as
 * bs_spec_sample without the workspace.  Limit: B * (2 * gamma + 1) <= bs_spec_sample_static_max_rows() (65536) logit
 * rows per call, BS_ESHAPE beyond that.  Calls no allocating routine.  All calls on one GPU share that GPU's array:
 * calls that overlap in time on the same GPU (different streams, different host threads) race; calls on one stream do
 * not.  The first call on a device looks the array's address up (a host-side lock, no stream work). */
size_t bs_spec_sample_static_max_rows(void);
int bs_spec_sample_static(const void* dev_target_logits, const void* dev_draft_logits,
                          const int32_t* dev_draft_tokens, int B, int gamma, int V, int dtype,
                          float temperature, const float* dev_uniforms, uint64_t seed, uint32_t round,
                          int32_t* dev_accept_len, int32_t* dev_next_token, float* dev_margins, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Arm selection (host only).  UCBSpec: Alg. 4 / its full version - arms 0..K-1 in order for the
 * first K rounds, then argmax of mean + (L/2) sqrt((1+n)/n^2 (1 + 2 ln(K t^2 sqrt(1+n)/delta))),
 * ties to the lowest index.  EXP3Spec: full version of Alg. 5 - eta_t = sqrt(ln K/(tK)),
 * p_t ~ exp(-eta_t * cumulative estimated loss), arm drawn by inverse CDF with the Philox uniform
 * (seed; 0, t-1, 0, 3); after the round Zhat = (L+1-y)/(L p_t[arm]).
 * y is the accepted length including the bonus token (Sec. 3), 1 <= y <= L+1 (a batch mean is fine).
 * ---------------------------------------------------------------------------------------------- */
typedef struct bs_bandit bs_bandit;
typedef enum { BS_UCBSPEC = 0, BS_EXP3SPEC = 1 } bs_bandit_kind;
int bs_bandit_create(int kind, int K, int L, double delta, uint64_t seed, bs_bandit** out);
int bs_bandit_destroy(bs_bandit* b);
int bs_bandit_select(bs_bandit* b, int* arm_out);
int bs_bandit_update(bs_bandit* b, int arm, double y); /* arm must be the last selected arm */
/* UCBSpec: the K indices mean+radius (+inf during round-robin); EXP3Spec: p_t for the next round. */
int bs_bandit_probs(bs_bandit* b, double* host_out_K);
/* pulls n_i, and per arm sum of y (UCBSpec) or cumulative estimated loss (EXP3Spec); rounds so far */
int bs_bandit_stats(bs_bandit* b, double* host_n_K, double* host_sum_K, int64_t* rounds_out);
/* Throughput as the reward (Sec. 6, second experiment: arms gamma in {0..L} incl. canonical decoding, the reward is the
 * round's throughput; the paper prints no formula, this normalisation is this library's and has no parity pin):
 *   y = 1 + L * min(1, (tokens / seconds) / ((L + 1) / canonical_seconds))
 * tokens = mean tokens the round emitted per sequence, seconds = its duration, canonical_seconds = duration of a
 * gamma = 0 round (one target pass).  The reference rate (L+1 tokens per target pass) bounds any arm, so y lies in
 * [1, L+1], the range bs_bandit_update and the confidence radius of Alg. 4 expect.
 * Errors: BS_EINVAL (NULL, non-positive times, negative tokens, L < 1). */
int bs_throughput_reward(double tokens, double seconds, double canonical_seconds, int L, double* y_out);
/* Reward of one round for a batch that shares one bandit (Alg. 3 with one arm per round for all sequences): the mean of
 * the accepted lengths y = host_n_emitted[b] over the sequences that took part in the round (entries > 0; a sequence
 * already at its goal, or skipped, reports 0 and is left out), so the value stays in [1, L+1].
 * host_n_emitted [B] int32 HOST memory (the copy of bs_spec_round's dev_n_emitted); n_active_out may be NULL.
 * Errors: BS_EINVAL (NULL, B < 1, a negative entry), BS_ESTATE (no entry > 0: there is no reward to feed back). */
int bs_batch_reward(const int32_t* host_n_emitted, int B, double* y_out, int* n_active_out);

/* ------------------------------------------------------------------------------------------------
 * Models (Sec. 2: a model is the conditional distribution softmax(logits/T); the network itself is
 * the workload's: pre-norm decoder, RMSNorm, RoPE on interleaved pairs, causal MHA/GQA, SwiGLU).
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff, vocab;
    int32_t dtype;          /* bs_dtype of matrices, embeddings, KV cache and stored activations */
    float rope_base;        /* e.g. 10000 */
    float norm_eps;         /* e.g. 1e-5 */
} bs_model_cfg;

typedef struct {
    const float* attn_norm; /* [d_model] */
    const void* wq;         /* [n_heads*head_dim, d_model] */
    const void* wk;         /* [n_kv_heads*head_dim, d_model] */
    const void* wv;         /* [n_kv_heads*head_dim, d_model] */
    const void* wo;         /* [d_model, n_heads*head_dim] */
    const float* ffn_norm;  /* [d_model] */
    const void* w_gate;     /* [d_ff, d_model] */
    const void* w_up;       /* [d_ff, d_model] */
    const void* w_down;     /* [d_model, d_ff] */
} bs_layer_weights;

typedef struct {
    const void* embed;              /* [vocab, d_model] */
    const float* final_norm;        /* [d_model] */
    const void* lm_head;            /* [vocab, d_model] */
    const bs_layer_weights* layers; /* host array of n_layers entries (copied by bs_model_create) */
} bs_model_weights;

typedef struct bs_model bs_model;
int bs_model_create(const bs_model_cfg* cfg, const bs_model_weights* dev_weights, bs_model** out);
int bs_model_destroy(bs_model* m);

/* Optional re-layout of a bf16 model's projection matrices and LM head for the verification pass (App. A: the
 * target scores gamma+1 positions at once, so every weight is read exactly once per pass and the pass runs at
 * the speed the weights stream from HBM).  The copy is cut into 64-row x 32-column blocks,
 * [rows/64][cols/32][4][64][8] bf16 with rows padded to 64, so that each matrix-core operand is one
 * contiguous kilobyte.  bs_model_packed_bytes: size of the copy, 0 if the model cannot be packed (fp32, or
 * d_model / n_heads*head_dim / d_ff not multiples of 32, or n_kv_heads*head_dim not a multiple of 16).
 * bs_model_pack: dev_buf is device memory of at least that size, 256-byte aligned, owned by the caller and
 * kept alive for the model's lifetime; the copy is enqueued on `stream` (a hipStream_t, NULL = default).
 * After it completes the model no longer reads the row-major projections (embedding and norm gains are still
 * read from the original pointers), so the caller may free them.  Results are bit-identical to the unpacked
 * model.  Errors: BS_EINVAL (NULL), BS_ESTATE (already packed), BS_ESHAPE, BS_EWORKSPACE. */
size_t bs_model_packed_bytes(const bs_model_cfg* cfg);
int bs_model_pack(bs_model* m, void* dev_buf, size_t bytes, void* stream);

/* KV cache bound to caller memory, model dtype, opaque to the caller.  Per layer K then V, each
 * [B][kv_head][rows][head_dim] with rows = max_len rounded up to 32; in a bf16 cache V is held transposed in
 * blocks of 32 keys ([rows/32][head_dim][32]) so that the matrix-core attention reads it without transposes. */
typedef struct bs_kv bs_kv;
size_t bs_kv_bytes(const bs_model_cfg* cfg, int B, int max_len);
int bs_kv_bind(const bs_model* m, int B, int max_len, void* dev_buf, size_t bytes, bs_kv** out);
int bs_kv_destroy(bs_kv* kv);

/* Workspace needed by bs_verify_forward / bs_prefill for at most max_rows = B*q_len query rows. */
size_t bs_forward_workspace_bytes(const bs_model_cfg* cfg, int B, int max_q_len, int max_len);

/* ------------------------------------------------------------------------------------------------
 * Target verification forward (App. A, the step that scores all gamma+1 positions of the draft block in one pass):
 * runs the model over q_len query tokens per sequence against its KV cache.
 *   query j of sequence b sits at position pos = kv_len[b] + j, attends to cache positions
 *   0..pos (causal), and its K/V are written to the cache at pos (the cache length itself is the
 *   caller's dev_kv_len; nothing else records it).
 *  dev_q_tokens [B, q_len] int32;  dev_kv_len [B] int32 (tokens already in the cache)
 *  logit_rows   how many trailing query rows per sequence get logits (q_len for verification,
 *               1 for a draft step, 0 for cache fill only)
 *  dev_logits   [B, logit_rows, vocab] float32 out (may be NULL if logit_rows == 0)
 * Sequences with kv_len[b] + q_len > max_len are skipped entirely and bit 0 of the device status
 * word (first int32 of the workspace) is set; other sequences are unaffected.  The library only ever ORs bits into that
 * word: zero it (the workspace once, say) before relying on it.
 * The same call serves the draft model's steps (q_len = 1 or 2, logit_rows = 1).  One or two rows in all (B * q_len <= 2)
 * of a small packed bf16 model with head_dim 64 run as ONE resident kernel of one workgroup per compute unit whose
 * workgroups wait for each other's outputs; it needs the GPU's compute units to itself while it runs (work of the same
 * stream or graph is ordered behind it anyway).  Passes of up to 16 rows per head group against a cache long enough for
 * several key splits combine the splits inside the attention kernel the same way (exchange cells in the workspace; only
 * when all workgroups of the launch fit on the device together, else a merge kernel runs instead; like the resident kernel
 * it counts on having the compute units to itself: other work running concurrently on other streams can make a wait run
 * into its bound).  Every wait is bounded: see bs_step_poll_limit.
 * ---------------------------------------------------------------------------------------------- */
int bs_verify_forward(const bs_model* m, const bs_kv* kv, const int32_t* dev_q_tokens,
                      const int32_t* dev_kv_len, int q_len, int logit_rows, float* dev_logits,
                      void* dev_workspace, size_t workspace_bytes, void* stream);
/* The bound of the waits inside kernels (the resident kernel's; the attention kernel's when it combines its key splits),
 * in polls of one cell (default 2^18, about a quarter of a second; 0 restores
 * the default).  A pass that runs out of polls ends without a result -- its logits and the cache rows it was to write are
 * not valid -- and sets bit 16 of the device status word; no launch ever waits without end.  Applies to passes enqueued
 * after the call.  Meant for tests of that path. */
int bs_step_poll_limit(unsigned polls);

/* Prompt processing: fills the cache for positions 0..n-1 of every sequence (same n for all), in
 * chunks through the same kernels.  dev_tokens [B, token_stride] int32, n <= token_stride.
 * dev_last_logits [B, vocab] float32 (logits after the last prompt token) or NULL. */
int bs_prefill(const bs_model* m, const bs_kv* kv, const int32_t* dev_tokens, int token_stride, int n,
               float* dev_last_logits, void* dev_workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * One speculative round for a batch (Alg. 2 with vanilla speculative decoding, App. A; the device part
 * of one iteration of Alg. 3).  An arm is a (draft model, gamma) pair; L = max gamma.
 * Device state owned by the caller and advanced by the round:
 *   dev_tokens [B, max_len] int32   the growing prompts (Alg. 3, pt_t)
 *   dev_total_len [B] int32         tokens per sequence; invariant: the target cache holds total_len-1
 *   dev_goal_len [B] int32          generation stops here (tokens beyond it are dropped; the reported
 *                                   accepted length is not truncated).  A round of speculation length gamma needs
 *                                   total_len + gamma <= max_len (its verification pass appends gamma+1 keys to a cache
 *                                   that holds total_len-1); a sequence for which that fails takes no part in the round:
 *                                   nothing is read or written for it, n_emitted is 0 and bit 8 of bs_round_status is
 *                                   set.  goal_len <= max_len - L therefore lets every arm run until the goal.
 * Random numbers: Philox(seed; b, t, slot, purpose) with t the device round counter (bs_round_reset).
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    const bs_model* target;
    const bs_kv* target_kv;
    int32_t n_drafts;
    const bs_model* const* drafts;     /* host array [n_drafts] */
    const bs_kv* const* draft_kvs;     /* host array [n_drafts], each bound with the same B, max_len */
    int32_t n_arms;
    const int32_t* arm_draft;          /* host array [n_arms]: index into drafts */
    const int32_t* arm_gamma;          /* host array [n_arms]: speculation length, >= 0; 0 = no draft tokens: the round is
                                          one step of canonical decoding (Alg. 1), y = 1 */
    int32_t B, max_len;
    int32_t* dev_tokens;
    int32_t* dev_total_len;
    const int32_t* dev_goal_len;
    float temperature;                 /* > 0, or 0 for greedy decoding (see bs_spec_sample) */
    uint64_t seed;
    void* dev_workspace;               /* bs_round_workspace_bytes(...) bytes, 256-byte aligned */
    size_t workspace_bytes;
    int32_t use_graph;                 /* 1: capture each arm's round once into a HIP graph and replay it */
    /* Draft-logit perturbation of the non-stationary workload (not in the paper; both 0 = none): every draft row
     * gets sigma * N(0,1) noise before it is drawn from, and the perturbed row is also the Q of the acceptance
     * test, so the round stays exact for the target distribution (Prop. 3.1 holds for any Q).  sigma =
     * noise_sigma[0] while floor(generated / noise_period) is even, noise_sigma[1] while it is odd
     * (noise_period 0: always noise_sigma[0]); generated = total_len[b] - prompt_len[b] at the start of the round.
     * Normals: Philox counter (b, t, draft position i, 4 + 8*g) gives four words for vocabulary ids 4g..4g+3;
     * (w0, w1) and (w2, w3) are Box-Muller pairs, radius from u1 = ((w>>8)+1) 2^-24, angle 2 pi (w>>8) 2^-24,
     * cosine first. */
    const int32_t* dev_prompt_len;     /* [B] int32 or NULL (= 0): tokens that were given rather than generated */
    float noise_sigma[2];
    int32_t noise_period;
} bs_round_cfg;

typedef struct bs_round bs_round;
size_t bs_round_workspace_bytes(const bs_model_cfg* target, const bs_model_cfg* const* drafts, int n_drafts,
                                int B, int L, int max_len);
int bs_round_create(const bs_round_cfg* cfg, bs_round** out);
int bs_round_destroy(bs_round* r);
/* Sets the device round counter t (enqueues a tiny kernel) and records that every draft cache holds the keys and
 * values of at least the first total_len-2 tokens of every sequence (true right after prefill of the same prompts).
 * From then on the library tracks how far each draft cache is valid: a draft model that was not selected for some
 * rounds never saw the tokens emitted meanwhile, and is brought up to date (passes of 16 tokens per sequence
 * through the same forward kernels, cache fill only) before its next proposal. */
int bs_round_reset(bs_round* r, uint32_t t0, void* stream);
/* Draft proposal alone (App. A, the gamma draws x~_i ~ Q(. | pt, x~_{<i})) for arm `arm` from the current device
 * state, without verification or commit: the round counter and the token state do not advance, and a following
 * bs_spec_round of the same arm repeats exactly these draws.  dev_draft_tokens [B, gamma] int32 and dev_draft_logits
 * [B, gamma, V] float32 (the rows of Q that were drawn from, after the perturbation if one is configured) may each
 * be NULL.  Not captured into a graph. */
int bs_draft_propose(bs_round* r, int arm, int32_t* dev_draft_tokens, float* dev_draft_logits, void* stream);
/* Enqueues draft proposal -> verification -> accept/reject -> commit for arm `arm`.
 *  dev_emitted   [B, L+1] int32 out: accepted draft tokens then the residual/bonus token
 *  dev_n_emitted [B] int32 out: y = tau + 1 (the reward of Sec. 3; 0 for sequences already at goal)
 * The caller copies dev_n_emitted to the host and synchronises before bs_bandit_update. */
int bs_spec_round(bs_round* r, int arm, int32_t* dev_emitted, int32_t* dev_n_emitted, void* stream);
/* Device status since the last bs_round_reset, OR of:
 *   1  a forward pass left out a sequence whose query rows would have run past max_len
 *   2  a token id outside [0, vocab) was replaced by 0
 *   4  total_len < 2 or > max_len at the start of a round (sequence left out)
 *   8  a sequence still generating had total_len + gamma > max_len (left out, see dev_goal_len above)
 *  16  a wait inside a kernel ran out of polls (bs_step_poll_limit): that round's tokens are not valid
 * Copies the word to *host_out (HOST memory) and WAITS for `stream`: this call synchronises.  Not for use while the
 * stream is being captured. */
int bs_round_status(bs_round* r, int32_t* host_out, void* stream);
/* Views into the round workspace for parity checks (valid after the round's stream work is done):
 * target logits [B, gamma+1, V] f32, draft logits [B, gamma, V] f32, draft tokens [B, gamma] int32,
 * margins [B, gamma] f32 of the most recent round. */
int bs_round_debug_views(bs_round* r, const float** dev_target_logits, const float** dev_draft_logits,
                         const int32_t** dev_draft_tokens, const float** dev_margins);

/* ------------------------------------------------------------------------------------------------
 * Measurement hook (not part of the method): while enabled, every launch of the bf16 weight-streaming
 * GEMM and of the bf16 attention kernel made OUTSIDE a graph capture carries its own start and stop
 * events (they take the begin and end times of the dispatch itself, so the elapsed time is the kernel's
 * alone).  bs_profile_collect synchronises on those events and returns, for launches of the asked
 * class, the summed kernel time in ms, the summed algorithmic bytes and the launch count.  Classes:
 * 1, 2, 4, 6, 8, 16 = GEMM launches with up to that many tiles of 16 activation rows (bytes: each weight element
 * once, N*K*2); 50 = the fused few-row projections of draft steps (same bytes); 60 = the whole-K projections with
 * fused epilogues that verification passes of up to 16 rows take on wide models (same bytes); 100 = attention (bytes
 * reported as 0: the cache lengths live on the device, the caller knows them); 0 = everything.
 * bs_profile_enable(1) starts an empty record; bs_profile_enable(0) stops recording and drops the record with its
 * events, so collect before switching off.  Events cannot be recorded into a stream capture: while the record is on, a
 * timed launch on a stream that is being captured fails with BS_ESTATE (switch the record off before capturing).  The
 * record is guarded by a mutex: launches, enable and collect may come from several host threads.
 * ---------------------------------------------------------------------------------------------- */
int bs_profile_enable(int on);
int bs_profile_collect(int row_tiles, double* host_total_ms, double* host_total_bytes, long long* host_launches);

#ifdef __cplusplus
}
#endif
#endif /* BANDITSPEC_H */
