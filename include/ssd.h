/* ssd.h -- C ABI of the MI355X (gfx950) library for the draft side of speculative
 * speculative decoding (SSD / Saguaro).
 *
 * What the calls compute is fixed by the paper: Alg. 1 (speculator loop:
 * predict_verify_outcomes, speculate_for_outcomes, cache lookup), Sec. 2.1
 * (verification: sequential acceptance, residual distribution, bonus token),
 * Sec. 4.1.1 (outcome prediction: top-F of the draft logits at each accept length,
 * without the token sent for verification), the definitions of speculation,
 * verification outcome and speculation cache (Sec. 2.1, Sec. 3.1), App. B (all
 * (K+1)F branches decoded together, each seeing the verified trunk and its own
 * path; the "glue" extend before each round; the once-per-round payload fields)
 * and App. C (token and cache-element counts).
 *
 * General conventions
 *   - Every function returns SSD_OK (0) or a negative ssd_status.  Nothing throws or
 *     aborts.  ssd_last_error() returns a thread-local message for the last failure.
 *   - Pointers named d_* are DEVICE memory, h_* are HOST memory.  Unless a comment says
 *     otherwise the caller owns them and must keep them alive until `stream` has reached
 *     the call.  Buffers inside ssd_model / ssd_ctx are owned by the library.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; none synchronises the host unless stated.
 *   - Branch row order (part of the contract): row = b (K+1) F + k F + j, with b the
 *     sequence, k the accept length 0..K and j the candidate rank 0..F-1.  With a fan-out
 *     F_0..F_K that differs per accept length (Sec. 4.1.2; ssd_ctx_create_fanout) rows run
 *     accept length by accept length: row = b R + (F_0 + .. + F_{k-1}) + j, j < F_k,
 *     R = F_0 + .. + F_K rows per sequence; wherever a layout below says [K+1][F], such a
 *     context holds [R] in that order (no padding).
 *   - Ordering of tokens wherever a maximum or a top-F is taken: larger score first,
 *     equal scores by smaller token id; NaN ranks below every number.
 *   - The library allocates device memory only in *_create; the hot calls
 *     (ssd_prespeculate, ssd_cache_lookup, ssd_ctx_commit, ssd_verify, ssd_verify_static,
 *     ssd_top_f, ssd_sample) allocate nothing.
 */
#ifndef SSD_H_
#define SSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SSD_OK = 0,
  SSD_EINVAL = -1,  /* null pointer, size out of range, shape the kernels do not support */
  SSD_ESTATE = -2,  /* call order: lookup before any pre-speculation, trunk not loaded, ... */
  SSD_EHIP = -3,    /* a HIP runtime call failed; message holds hipGetErrorString */
  SSD_ENOMEM = -4   /* device allocation failed */
} ssd_status;

enum { SSD_F32 = 0, SSD_BF16 = 1 };

/* Limits of this build. */
enum { SSD_MAX_F = 16, SSD_MAX_K = 15 };

typedef struct ssd_model ssd_model; /* decoder weights, library-owned device copies */
typedef struct ssd_ctx ssd_ctx;     /* per-batch state: trunk KV, branch KV, speculation cache */

/* A Llama-style decoder (RMSNorm, rotary embedding pairing (i, i + head_dim/2), grouped-query
 * attention, SwiGLU), the family of the paper's draft and target models (Sec. 4 "Setup"). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype;          /* SSD_F32 or SSD_BF16: storage type of weights and KV.  Arithmetic
                             accumulates in fp32 either way; logits are always fp32. */
  float rope_theta, rms_eps;
  int32_t tie_embeddings; /* 1: the LM head is the embedding matrix */
} ssd_model_config;

/* Weights as the linear layers apply them, row-major [out_features][in_features], elements of
 * config.dtype (bf16 = the upper 16 bits of the fp32 pattern).  All pointers are DEVICE memory;
 * the per-layer members are HOST arrays of n_layers device pointers.  ssd_model_create copies
 * (and re-tiles) everything on `stream`; the caller may free its buffers once that stream has
 * been synchronised. */
typedef struct {
  const void* d_embed;      /* [vocab][d_model] */
  const void* d_lm_head;    /* [vocab][d_model], NULL when tie_embeddings */
  const void* d_final_norm; /* [d_model] */
  const void* const* h_attn_norm; /* [d_model] each */
  const void* const* h_wq;        /* [n_q_heads*head_dim][d_model] */
  const void* const* h_wk;        /* [n_kv_heads*head_dim][d_model] */
  const void* const* h_wv;        /* [n_kv_heads*head_dim][d_model] */
  const void* const* h_wo;        /* [d_model][n_q_heads*head_dim] */
  const void* const* h_mlp_norm;  /* [d_model] */
  const void* const* h_w_gate;    /* [d_ffn][d_model] */
  const void* const* h_w_up;      /* [d_ffn][d_model] */
  const void* const* h_w_down;    /* [d_model][d_ffn] */
} ssd_model_weights;

/* Shape of the pre-speculation round: speculative lookahead K and uniform fan-out F
 * (Sec. 2.1 Def. "speculation"; Sec. 4.1.1 Def. "fan-out"). */
typedef struct {
  int32_t batch;     /* B >= 1 sequences */
  int32_t K;         /* 1..SSD_MAX_K drafted tokens per speculation = decode steps per branch */
  int32_t F;         /* 1..SSD_MAX_F bonus-token candidates per accept length */
  int32_t max_trunk; /* capacity of the trunk KV in positions, per sequence */
  int32_t flags;     /* 0, or SSD_CTX_* bits: which kernels serve the context (results are the same to rounding) */
  int32_t kv_pages;  /* 0: every sequence owns max_trunk trunk positions.  n >= 2: paged trunk (App. B, the paged attention and
                        block tables of the paper's system): per layer one pool of n pages of 32 positions, shared by the
                        sequences, each reaching its positions through its row of a block table; page 0 is the all-zero
                        page every unmapped block points at and is never handed out.  Fused contexts only, max_trunk <=
                        16384 (it then only sizes the block table).  Same bits as the contiguous trunk. */
} ssd_round_config;

/* ssd_round_config.flags.  By default a context whose model and shape the fused decode pass supports (bf16, head_dim 64)
 * runs every batched forward as one persistent kernel. */
enum {
  SSD_CTX_PER_OPERATOR = 1, /* never the fused pass: one kernel per operator */
  SSD_CTX_FUSED_PHASES = 2, /* the fused pass as one launch per phase instead of one persistent launch: no grid barrier, so
                               no need for all its workgroups to be resident at once; same bits as the persistent launch */
  SSD_CTX_NARROW_PASSES = 4, /* a context with more than 48 rows in a batched forward runs them as passes of whole sequences
                                of at most 48 rows (the weights are then streamed once per pass) instead of wide passes of
                                up to 384 rows; a comparison aid */
  /* Precision of the activations the narrow fused pass hands from phase to phase.  The three that meet the weights (the
   * normalised residual stream xn, the attention output att, the SwiGLU output act) travel in fp16 and the linear
   * layers multiply them with fp16 copies of the bf16 weights (exact for |w| >= 2^-14, absolute error <= 2^-25 below;
   * activations beyond +-65504 saturate); the rotated queries q and the softmax probabilities p meet the bf16 KV store
   * and are bf16.  A tensor is one 16-bit plane or two (head + remainder: about twice the significant bits, twice the
   * operand traffic and MFMAs).  Default: xn, att, act one fp16 plane (11 bits), q and p two bf16 planes; measured
   * against a float64 reference through the 16 layers of the 1B shape: 2.6e-3 (worst row).
   * SSD_CTX_TWO_PLANES: every tensor two planes unless its ONE_PLANE bit is set (alone: 1.1e-3, at +4 % time on a 24-row
   * step and +11 % on a 48-row step at 8192 keys).  ONE_PLANE_Q / ONE_PLANE_P: that tensor as one bf16 plane too (with
   * both, = ONE_PLANE_ALL: 1.1e-2 and no faster than the default).  Wide passes always carry xn, att, act as one plane.
   * EINVAL for a combination the narrow pass is not compiled for: compiled are the default and TWO_PLANES alone; others
   * are a build option (-DSSD_FUSED_PLANE_MASKS="X(0) X(7) X(31)", bit i of a mask = tensor i as one plane). */
  SSD_CTX_ONE_PLANE_XN = 0x100, SSD_CTX_ONE_PLANE_ATT = 0x200, SSD_CTX_ONE_PLANE_ACT = 0x400,
  SSD_CTX_ONE_PLANE_Q = 0x800, SSD_CTX_ONE_PLANE_P = 0x1000, SSD_CTX_ONE_PLANE_ALL = 0x1f00,
  SSD_CTX_TWO_PLANES = 0x2000
};

/* Read-only device views of the context's state, for tests and for the verifier's payload. */
typedef struct {
  const int32_t* d_trunk_len;  /* [B] positions currently in the trunk */
  const int32_t* d_keys;       /* [B][K+1][F] cached bonus tokens (cache keys) */
  const int32_t* d_tokens;     /* [B][K+1][F][K] speculation per cached outcome */
  const float* d_logits;       /* [B][K+1][F][K][V] logits each of those tokens was drawn from */
  const float* d_hidden;       /* [B][K+1][F][K][d_model] final-norm hidden states */
  const float* d_glue_logits;  /* [B][K+1][V] logits of the glue extend */
  const float* d_glue_hidden;  /* [B][K+1][d_model] */
  const void* const* h_trunk_k; /* host array [n_layers] of device [B][max_trunk][Hkv][D] (model dtype) */
  const void* const* h_trunk_v; /* same layout (both null-free but not meaningful to read in a paged context).  Contexts served by the fused decode pass (bf16, head_dim 64, at most 48
                                   rows per pass) keep both head-major with T = max_trunk rounded up to 64: keys
                                   [B][Hkv][T][D], values transposed per 32-position block [B][Hkv][T/32][D][32] */
  int32_t batch, K, F, vocab, d_model, max_trunk;
  int32_t fused_pass;          /* 0: one kernel per operator; 1: fused pass, one launch per phase; 2: one persistent launch */
  int32_t pass_rows;           /* most rows of one fused pass: 48 (narrow passes), 384 (wide passes), 0 without the fused pass */
} ssd_views;

const char* ssd_last_error(void);

/* ---- set-up (not on the hot path; these allocate) ------------------------------------------ */

int ssd_model_create(const ssd_model_config* cfg, const ssd_model_weights* w, void* stream, ssd_model** out);
/* A random-init model generated on the device (the synthetic stand-in for trained weights, at any size: no host
 * copy exists).  Every matrix element is N(0, 0.02)-like, every RMSNorm gain 1, from integer arithmetic alone, so the
 * host-side generator the tests use gives the same bits: element i (row-major [out][in]) of tensor t is
 * float(S - 131070) * float(0.02 / 37837.227...), S = the sum of the four 16-bit lanes of
 * mix64(mix64(seed + 0x9E3779B97F4A7C15 (t + 1)) + i) (mix64 = the SplitMix64 finaliser), rounded to bf16
 * (nearest even) for bf16 models.  Tensor ids: 0 embedding, 1 LM head (untied models), 16 + 16 l + {0 wq, 1 wk, 2 wv, 3 wo,
 * 4 w_gate, 5 w_up, 6 w_down} for layer l.  Runs on `stream` and SYNCHRONISES it before returning. */
int ssd_model_create_random(const ssd_model_config* cfg, uint64_t seed, void* stream, ssd_model** out);
int ssd_model_destroy(ssd_model* m);
/* A bf16 model whose shape the fused passes take holds every linear layer twice: in the order the fused passes stream
 * it, and in the tile order of the per-operator kernels (contexts with SSD_CTX_PER_OPERATOR, or round shapes the fused
 * passes do not take).  A caller that only creates fused contexts gives the second copy back (2.47 GB at the 1B shape):
 * afterwards a context that would need it fails with ESTATE.  ESTATE also while such a context is alive, and for models
 * the fused passes do not take (they have no other copy).  Synchronises the device.  Idempotent. */
int ssd_model_release_operator_weights(ssd_model* m);

/* The context keeps a pointer to `model`; destroy the context first. */
int ssd_ctx_create(const ssd_model* model, const ssd_round_config* cfg, ssd_ctx** out);
int ssd_ctx_destroy(ssd_ctx* ctx);

/* Cache shape (Sec. 4.1.2, Theorem "Geometric Fan-Out"): a context whose fan-out differs per accept length.
 * h_fanout: host int32 [K+1], F_k in 1..SSD_MAX_F (read during the call only); cfg->F is ignored.  Everything else
 * is as for ssd_ctx_create; ssd_views.F reports the largest F_k.  ssd_ctx_fanout copies F_0..F_K of any context
 * to h_fanout [K+1]. */
int ssd_ctx_create_fanout(const ssd_model* model, const ssd_round_config* cfg, const int32_t* h_fanout, ssd_ctx** out);
int ssd_ctx_fanout(const ssd_ctx* ctx, int32_t* h_fanout);

/* The theorem's shape as integers (host only, no GPU work): for a speculator with acceptance rate a in (0,1) whose
 * cache-miss rate at fan-out F is F^-r (r > 0), F_k proportional to a^(k/(1+r)) below K and the last one larger by
 * (1-a)^(-1/(1+r)), scaled so that F_0 + .. + F_K = budget (the closed form of F_0 in the theorem's proof).
 * The paper leaves the step to integers open; here every F_k is kept within 1..f_max (a bound that binds holds that
 * F_k, the others share the rest in the same proportions), shares are rounded down and the units left over go to
 * the largest fractional parts, lower k first on ties.  out h_fanout int32 [K+1].
 * EINVAL unless K+1 <= budget <= (K+1) f_max. */
int ssd_geometric_fanout(int32_t budget, int32_t K, double a, double r, int32_t f_max, int32_t* h_fanout);

/* Trunk := KV of d_tokens[b][0 .. h_lens[b]-1] (row stride `stride` tokens), computed with the same
 * extend kernels in chunks.  EINVAL if a length exceeds max_trunk - (2K+2). */
int ssd_ctx_prefill(ssd_ctx* ctx, const int32_t* d_tokens, int32_t stride, const int32_t* h_lens, void* stream);
/* Trunk := given KV (a synthetic prefix standing in for a prefill).  d_k, d_v:
 * [n_layers][B][len][n_kv_heads][head_dim] in the model dtype; every sequence gets length `len`. */
int ssd_ctx_load_trunk(ssd_ctx* ctx, const void* d_k, const void* d_v, int32_t len, void* stream);
/* Trunk of sequence b := h_lens[b] positions of synthetic KV (a stand-in for a prefill that is not on the measured path),
 * generated on the device with the hash of ssd_model_create_random and unit variance: element (position t, KV head h,
 * dim d) of sequence b has index (b << 40) + (t n_kv_heads + h) head_dim + d in tensor (1 << 20) + 2 l (keys of layer l) or
 * (1 << 20) + 2 l + 1 (values).  h_lens: host int32 [B], each >= 1 and <= max_trunk - (2K+2).  Synchronises `stream`. */
int ssd_ctx_fill_synthetic_kv(ssd_ctx* ctx, const int32_t* h_lens, uint64_t seed, void* stream);
/* Trunk of sequence b := its first h_lens[b] positions (1 <= h_lens[b] <= the context's current bound of the trunk
 * lengths; host int32 [B], read during the call): a batch of different prefix lengths from one loaded or prefilled
 * block, or a rollback.  EINVAL if a length is out of range.  Synchronises `stream`. */
int ssd_ctx_truncate_trunk(ssd_ctx* ctx, const int32_t* h_lens, void* stream);

/* Paged contexts and continuous batching (App. B).  Pages are taken when a call is about to write positions a sequence
 * has no page for (prefill, load, and the glue extend of a round: up to the host's bound of the trunk length + K+1) and
 * handed back by the calls that synchronise: ssd_ctx_refresh_bounds (page rollback: pages wholly behind a sequence's
 * verified text, i.e. rejected positions and bounds that ran ahead), ssd_ctx_truncate_trunk, ssd_ctx_release_sequence.
 * ENOMEM when the pool is empty: the context is unchanged apart from pages already taken for the same call; release a
 * sequence or refresh the bounds and call again.
 * ssd_ctx_prefill runs all sequences in common passes up to the longest prompt, so until it returns every sequence holds
 * pages for that length (the surplus goes back at its end): a pool sized for the true lengths only is filled slot by slot
 * with ssd_ctx_prefill_sequence.  The block table lives in pinned host memory and is copied to the device in stream
 * order whenever it changed; calls on one context are not thread-safe.
 *   ssd_ctx_kv_pages          total pages (0 for a contiguous trunk) and pages currently free.
 *   ssd_ctx_release_sequence  sequence b finished: its pages return to the pool and its trunk is empty; a round must not
 *                             run before the slot is refilled (ESTATE from ssd_prespeculate: empty trunk).  Synchronises.
 *   ssd_ctx_prefill_sequence  slot b := KV of d_tokens[0 .. len-1] (device int32), computed by extend passes over that one
 *                             sequence while the other slots keep their state: the join of a new request.  Works for
 *                             contiguous contexts too.  The speculation cache is dropped.  Synchronises. */
int ssd_ctx_kv_pages(const ssd_ctx* ctx, int32_t* total, int32_t* free_pages);
int ssd_ctx_release_sequence(ssd_ctx* ctx, int32_t b, void* stream);
int ssd_ctx_prefill_sequence(ssd_ctx* ctx, int32_t b, const int32_t* d_tokens, int32_t len, void* stream);

/* ---- hot path --------------------------------------------------------------------------------- */

/* One pre-speculation round (Alg. 1: predict_verify_outcomes + speculate_for_outcomes; App. B).
 *   d_pending      int32 [B][K+1] = {last verified token, s_1..s_K}: the speculation now being verified.
 *   d_temperature  float [B]; 0 = greedy.  T > 0: each branch token is argmax(logit/T + Gumbel) with
 *                  noise from the counter-based generator keyed (round_seed, stream 2, row, step, token).
 * Steps enqueued on `stream`: glue extend of the pending block onto the trunk (KV slots
 * trunk_len .. trunk_len+K, logits z_1..z_{K+1}); fan-out keys[b][k][:] = top-F of z_{k+1} without
 * s_{k+1} (nothing excluded at k = K); K batched decode steps over all B(K+1)F rows, row (b,k,j)
 * starting from keys[b][k][j] at position trunk_len+1+k and seeing trunk[0 .. trunk_len+k] plus its own
 * tokens; tokens and logits of every step go straight into the speculation cache.
 * trunk_len itself is not changed (see ssd_ctx_commit).  ESTATE if the trunk is empty or the host's
 * upper bound of trunk_len + 2K+2 exceeds max_trunk. */
int ssd_prespeculate(ssd_ctx* ctx, const int32_t* d_pending, const float* d_temperature, uint64_t round_seed,
                     void* stream);

/* Teacher forcing for parity tests: when set, branch row inputs are taken from the caller instead of
 * the library's own selection/sampling (outputs are still written as usual).  d_keys [B][K+1][F] feeds
 * step 0, d_tokens [B][K+1][F][K] entry i-1 feeds step i.  Either may be NULL (not forced).  The context keeps the
 * POINTERS, not copies: both arrays stay caller-owned and must remain valid until they are replaced or cleared and every
 * ssd_prespeculate enqueued meanwhile has run. */
int ssd_ctx_set_forced(ssd_ctx* ctx, const int32_t* d_keys, const int32_t* d_tokens);

/* Saguaro sampling scheme sigma_{F,C} (Sec. 4.2.1): with C < 1 every later ssd_prespeculate draws the branch tokens of
 * sampled sequences (temperature > 0) from the step's logits with its own top-F entries lowered by T log(1/C), and the
 * cache holds those lowered logits (the distribution a verifier must be given).  The fan-out keys always rank the
 * model's own logits; greedy sequences are unaffected.  C in [0, 1]; 1 (the default) switches the scheme off.
 * Host-only call, takes effect from the next round. */
int ssd_ctx_set_saguaro(ssd_ctx* ctx, float C);

/* Look the realised verification outcome up (Alg. 1; payload fields of App. B).
 *   in : d_accept_len int32 [B] (k in 0..K), d_bonus int32 [B] (t*)
 *   out: d_hit uint8 [B] (1 = cache hit), d_branch int32 [B] (rank j of the hit, -1 on a miss),
 *        d_spec_tokens int32 [B][K] (the cached speculation; -1 on a miss),
 *        d_logits_ptr (optional) const float* [B]: device address of the hit's [K][V] logits, NULL on a miss.
 * An accept length outside 0..K counts as a miss.  ESTATE before the first ssd_prespeculate. */
int ssd_cache_lookup(ssd_ctx* ctx, const int32_t* d_accept_len, const int32_t* d_bonus, uint8_t* d_hit,
                     int32_t* d_branch, int32_t* d_spec_tokens, const float** d_logits_ptr, void* stream);

/* After the outcome (k, t*) (Alg. 1: the speculator appends the accepted tokens; App. B "Glue & Recurrence" and the
 * rollback of rejected tokens' cache pages there): trunk_len[b] += k+1, which keeps the glue positions of the last
 * verified token and the k accepted ones and drops the rest.  Values of d_accept_len are clamped to 0..K. */
int ssd_ctx_commit(ssd_ctx* ctx, const int32_t* d_accept_len, void* stream);

/* Lossless verification (Sec. 2.1), stateless, meant for a stream of its own.
 *   d_target_logits float [B][K+1][V]: row i = target distribution of the token after s_1..s_i.
 *   d_draft_logits  float [B][K][V]:   row i = distribution s_{i+1} was drawn from (may be NULL if every
 *                                      temperature is 0).
 *   d_spec_tokens int32 [B][K];  d_temperature float [B] (0 = greedy).
 * T = 0: accept while argmax(target row i) == s_{i+1}; bonus = argmax of the first mismatching row (row K
 * if none).  T > 0: p = softmax(target/T), q = softmax(draft/T) in fp64; accept s_{i+1} iff u_i q(s) < p(s)
 * with u_i from generator stream 0 keyed (seed, b, i, 0); bonus = argmax_t log(max(p_t - q_t, 0)) + g_t at
 * the first rejected row (residual distribution), or argmax_t log p_t + g_t at row K, g from stream 1 keyed
 * (seed, b, k, t).  A residual without mass falls back to p.
 *   out: d_accept_len int32 [B], d_bonus int32 [B].
 *   d_workspace: device scratch of ssd_verify_workspace_bytes(B, K) bytes, 16-byte aligned, private to the call until
 *   `stream` has passed it (every pass over a row of logits is shared among several workgroups, whose partial
 *   results meet there).
 * EINVAL for B < 1, K < 1 or K > SSD_MAX_K, V < 2, null pointers. */
int ssd_verify(const float* d_target_logits, const float* d_draft_logits, const int32_t* d_spec_tokens,
               const float* d_temperature, int32_t B, int32_t K, int32_t V, uint64_t seed,
               int32_t* d_accept_len, int32_t* d_bonus, void* d_workspace, void* stream);
size_t ssd_verify_workspace_bytes(int32_t B, int32_t K);

/* ssd_verify for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error behaviour as ssd_verify, without
 * d_workspace: the partial results of the passes meet in a static device array of ssd_verify_static_capacity() bytes
 * (1 MiB; every GPU the library runs on holds one until the process ends).  The call allocates nothing, neither with
 * hipMalloc nor through any library.  EINVAL if ssd_verify_workspace_bytes(B, K) exceeds the capacity (B (2K+1) up to
 * about 1200 rows of logits fit).  All calls on one GPU share that GPU's array: two calls whose work overlaps in time on
 * one GPU (different streams, or different threads) race; calls on one stream are ordered and safe.  Nothing in the array
 * has to be cleared between calls. */
int ssd_verify_static(const float* d_target_logits, const float* d_draft_logits, const int32_t* d_spec_tokens,
                      const float* d_temperature, int32_t B, int32_t K, int32_t V, uint64_t seed,
                      int32_t* d_accept_len, int32_t* d_bonus, void* stream);
size_t ssd_verify_static_capacity(void);

/* The low-latency backup speculator of the fallback strategy (Sec. 4.3: after a cache miss at large batch the
 * next speculation is K random tokens).  out d_tokens int32 [B][K]: token i of sequence b is the 64-bit hash
 * (seed, stream 4, b, i, 0) of the library's counter-based generator modulo V, uniform over the vocabulary.  Their
 * verification at temperature > 0 takes the uniform distribution as the draft's, i.e. all-zero draft logits. */
int ssd_backup_random(uint64_t seed, int32_t B, int32_t K, int32_t V, int32_t* d_tokens, void* stream);

/* The selection kernel on caller-provided logits (Sec. 4.1.1).  d_logits float [rows][V] with row stride
 * `ld` elements; d_exclude int32 [rows] token to skip per row, or -1 (d_exclude may be NULL);
 * out d_ids int32 [rows][F].  d_workspace: NULL (one workgroup per row), or ssd_top_f_workspace_bytes(rows) of device
 * memory (8-byte aligned, contents irrelevant, private to the call until `stream` has passed it): few rows of a large
 * vocabulary are then shared among several workgroups each, with the same result.  EINVAL if F > SSD_MAX_F or
 * F + 1 > V. */
int ssd_top_f(const float* d_logits, int64_t ld, const int32_t* d_exclude, int32_t rows, int32_t V, int32_t F,
              int32_t* d_ids, void* d_workspace, void* stream);
size_t ssd_top_f_workspace_bytes(int32_t rows);

/* The branch sampler on caller-provided logits: d_out[r] = argmax_t logits[r][t] (T[r] == 0) or
 * argmax_t logits[r][t]/T[r] + g(seed, stream 2, row_base + r, step, t) in fp64.  d_temperature float [rows]. */
int ssd_sample(const float* d_logits, int64_t ld, const float* d_temperature, int32_t rows, int32_t V,
               uint64_t seed, int32_t row_base, int32_t step, int32_t* d_out, void* stream);
/* Test aid: the same draw with every token of a sampled row scored in fp64 (ssd_sample scans in fp32 and scores in fp64
 * only the tokens within the fp32 error bound of the maximum; both must give the same token). */
int ssd_sample_fp64_scan(const float* d_logits, int64_t ld, const float* d_temperature, int32_t rows, int32_t V,
                         uint64_t seed, int32_t row_base, int32_t step, int32_t* d_out, void* stream);

/* ---- generic extend (the glue step on its own; also how a target model is run) ------------------ */

/* Forward T tokens per sequence at positions trunk_len+offset .. +T-1 (causal among themselves, seeing
 * trunk[0 .. trunk_len+offset-1]); writes their KV into those trunk slots and, if d_logits is not NULL,
 * their logits to d_logits [B][T][V].  trunk_len is unchanged.  T <= K+1. */
int ssd_ctx_extend(ssd_ctx* ctx, const int32_t* d_tokens, int32_t T, int32_t offset, float* d_logits, void* stream);

/* The host keeps only an upper bound of trunk_len (it grows by K+1 per commit, since accept lengths live on the
 * device).  This call SYNCHRONISES `stream`, reads the true lengths back and tightens the bound; use it between
 * rounds of a long generation, never inside the hot path.  EHIP if a bounded wait of the fused pass has expired
 * (see ssd_ctx_status). */
int ssd_ctx_refresh_bounds(ssd_ctx* ctx, void* stream);

/* Health of a context served by the persistent fused pass.  That kernel separates its phases by grid barriers, which
 * complete only while all its workgroups are resident at once.  The library checks at ssd_ctx_create that they fit the
 * device and makes every persistent launch of the process wait (on the device) for the previous one wherever that ran on
 * another stream; a kernel of the caller's own that occupies compute units for seconds could still starve a barrier.
 * Every wait inside the kernel is bounded: on expiry the kernel sets a word in pinned host memory and ends.  From then
 * on the context's barrier state and everything computed since are invalid, and ssd_prespeculate, ssd_cache_lookup,
 * ssd_ctx_commit, ssd_ctx_extend, ssd_ctx_prefill, ssd_ctx_refresh_bounds and ssd_ctx_read_timing return SSD_EHIP as soon
 * as the host sees the word (calls enqueued before that have returned SSD_OK: check ssd_ctx_status after synchronising
 * when in doubt).
 *   ssd_ctx_status   non-blocking, no GPU work: SSD_OK, or SSD_EHIP once a wait has expired.
 *   ssd_ctx_recover  SYNCHRONISES the device, rebuilds the barrier state, clears the fault and invalidates the
 *                    speculation cache; trunk_len is kept, the trunk's contents behind it may be partly written
 *                    (the next glue extend rewrites them). */
int ssd_ctx_status(const ssd_ctx* ctx);
int ssd_ctx_recover(ssd_ctx* ctx);

/* Test aids for contexts served by the fused pass (ESTATE elsewhere); never needed in production.
 *   SSD_DEBUG_BARRIER_EPOCH  the grid barrier numbers its barriers on from launch to launch in 32 bits; restart the
 *                            count at `value` (SYNCHRONISES the device), e.g. shortly before the wrap.
 *   SSD_DEBUG_SPIN_LIMIT     polls a bounded wait takes before it gives up (0 = the default, seconds of wall time): a
 *                            tiny value makes the waits of the next launches expire, which is how the error path is
 *                            tested without ever hanging a kernel. */
enum { SSD_DEBUG_BARRIER_EPOCH = 1, SSD_DEBUG_SPIN_LIMIT = 2 };
int ssd_ctx_debug_set(ssd_ctx* ctx, int32_t what, uint32_t value);

/* Measurement aid.  With timing on, ssd_prespeculate records HIP events on its stream around the glue extend,
 * the fan-out and each of the K branch-decode steps.  ssd_ctx_read_timing waits for the last event of the most
 * recent round and returns h_ms[K+2] = {glue, fan-out, step 0 .. step K-1} in milliseconds.  In a context served by
 * the fused decode pass n may also be 2K+2: the last K entries are then the durations of the fused kernel alone in
 * each step (events recorded on `stream` right around its launch).  Enabling creates the events (set-up, not hot
 * path). */
int ssd_ctx_enable_timing(ssd_ctx* ctx, int32_t on);
int ssd_ctx_read_timing(ssd_ctx* ctx, float* h_ms, int32_t n);

/* Measurement aid for contexts served by the fused decode pass (bf16 model, at most 48 rows per pass): with phase
 * clocks on, every workgroup of the persistent kernel records the device's 100 MHz real-time counter at the entry of
 * each phase (slot 0), after the grid barrier in front of it (1) and at the end of its work (2); slots 3..7 are
 * probes inside some phases (unused slots keep their last value).  ssd_ctx_read_phase_clocks
 * SYNCHRONISES the device and copies the clocks of the most recent pass to h_ticks[phase][8][workgroup]
 * (n = capacity in entries; *n_phases and *n_workgroups receive the extents; phases: 0 embedding, then per layer
 * {qkv, attention partials, attention merge, o-proj, gate/up, down}, last the LM head).  ESTATE in other contexts. */
int ssd_ctx_enable_phase_clocks(ssd_ctx* ctx, int32_t on);
int ssd_ctx_read_phase_clocks(ssd_ctx* ctx, uint64_t* h_ticks, int64_t n, int32_t* n_phases, int32_t* n_workgroups);

int ssd_ctx_views(const ssd_ctx* ctx, ssd_views* out);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H_ */
