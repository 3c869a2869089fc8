/*
 * sr.h -- C boundary of the selective-rollout decode library for AMD MI355X (gfx950).
 *
 * The library runs the group-batched multi-turn rollout of one GRPO step and the
 * Selective-Rollout gate that retires converged groups mid-batch:
 *
 *   - G samples per prompt ("group") advance one environment step ("turn") at a time;
 *     each turn an observation chunk is appended to every live sequence and an action
 *     is decoded token by token (paper Section 2.2 and Appendix C.1/C.2: token layout
 *     [prompt, o_1, a_1, o_2, a_2, ...], one model call per step per trajectory);
 *   - after turn K the mean pairwise prefix edit distance d_K of each group's action
 *     sequences (Section 3.2) is compared with the threshold d_L and a group is cut iff
 *     d_K < d_L (Eq. 2); a cut group stops generating and leaves the batch (Section 3.2,
 *     paragraph "The gate"; Appendix C.1).
 *
 * Conventions
 *   - Every function returns SR_OK (0) or a negative sr_status; nothing throws or exits.
 *   - "device" pointers are HIP device memory of the current device; "host" pointers are
 *     ordinary host memory.  The caller owns every buffer it passes in.  The library owns
 *     its packed weight copy, the KV page pool, page tables, the action table and all
 *     scratch; they are released by sr_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream unless stated otherwise.  One context must be driven
 *     from one stream at a time.  Page tables and row maps reach the device through pinned
 *     staging slots guarded by events, so sr_prefill_chunk, sr_decode_step, sr_gate and
 *     sr_finish_sequences do not wait for the stream; sr_retire_and_compact waits once, for
 *     the retire mask (the page allocator lives on the host).
 *   - Batch rows are ordered group-major: while no sequence has finished early, live row r
 *     belongs to live group r / G, member r % G.  Retirement removes whole groups,
 *     sr_finish_sequences single members; both keep the order of the survivors
 *     (sr_get_live_map names the original sequence of every row).
 *   - All live sequences have the same length at all times (lock-step turns).
 *   - bf16 tensors are raw 16-bit patterns; matrices are row-major [out_features][in_features].
 */
#ifndef SR_H
#define SR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SR_OK = 0,
    SR_E_ARG = -1,    /* null pointer, bad shape, turn out of range, chunk_len <= 0, G < 2, ... */
    SR_E_NOMEM = -2,  /* KV page pool exhausted (checked on the host before any launch) or allocation failed */
    SR_E_STATE = -3,  /* call out of order: decode before prefill, gate with too few recorded actions, ... */
    SR_E_HIP = -4,    /* a HIP runtime call failed; sr_strerror gives the text */
    SR_E_LIMIT = -5   /* a size beyond the fixed capacity of an entry point that allocates nothing */
} sr_status;

typedef struct sr_ctx sr_ctx;

/* Decoder shape: pre-norm blocks, RMSNorm, rotate-half RoPE, grouped-query attention,
 * SwiGLU FFN.  head_dim must be 64 or 128; n_q_heads % n_kv_heads == 0.  (The paper names the
 * model family only -- Section 3.1; these fields describe any decoder of that family.) */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rms_eps, rope_theta;
    int32_t qkv_bias;     /* 1: q/k/v projections add a bias vector */
    int32_t tied_lm_head; /* 1: the LM head is the embedding matrix (sr_weights.lm_head is ignored and may be
                             NULL); 0: a separate [vocab][hidden] matrix */
} sr_model_shape;

typedef struct {
    int32_t page_tokens;     /* tokens per KV page: 32, 64 or 128 */
    int32_t max_seq_len;     /* longest context any sequence will reach */
    int32_t max_turns;       /* width of the per-sequence action table */
    int32_t action_mod;      /* action id of a turn = (first decoded token of the turn) % action_mod;
                                0 = the host supplies action ids with sr_set_actions */
    int32_t max_prefill_rows;/* rows (sequences x chunk tokens) processed per prefill pass; 0 = default 8192 */
    uint64_t kv_pool_bytes;  /* size of the KV page pool (K and V, all layers) */
    float temperature;       /* 0 = greedy decoding; > 0 = sample from softmax(logits / temperature) (the paper's
                                rollouts use 0.7, Section 3.1) by the Gumbel-max rule:
                                token = argmax_v (logit_v / T - ln(-ln(u_v))), lowest index on ties, with
                                u_v = (top 23 bits of SplitMix64(key, counter v) + 0.5) / 2^23 and key derived from
                                (sample_seed, original sequence id, position of the token): reproducible, and
                                independent of where the sequence sits in the batch */
    uint64_t sample_seed;
    float tau_H;             /* 0 = the one-clause gate of Eq. 2; > 0 = sr_gate also retires a group when the
                                fraction of its members that have finished (sr_finish_sequences) is >= tau_H
                                (Appendix E, Eq. 3) */
    int32_t fp32_debug;      /* 1 = debugging build of the path: every activation, the stored keys and values
                                and the attention probabilities stay in single precision (weights are the same
                                bf16 values, widened exactly) and the contractions run as plain fp32
                                multiply-adds.  Paging, copy-on-write, the split of the context and of the
                                projections' inner dimension, the order in which partial results are added,
                                token selection, gate and compaction are the ones of the normal path, so a
                                difference from an exact evaluation beyond single-precision rounding (logits:
                                1e-4) points at indexing rather than at bf16 operands.  Slow; a KV page takes
                                twice the bytes, so kv_pool_bytes holds half as many pages. */
} sr_options;

/* bf16 device pointers; borrowed only for the duration of sr_load_weights. */
typedef struct {
    const void *wq, *wk, *wv;   /* [n_q*d][hidden], [n_kv*d][hidden], [n_kv*d][hidden] */
    const void *wo;             /* [hidden][n_q*d] */
    const void *wg, *wu;        /* [ffn][hidden] */
    const void *wd;             /* [hidden][ffn] */
    const void *bq, *bk, *bv;   /* [n_q*d], [n_kv*d], [n_kv*d]; ignored when qkv_bias == 0 */
    const void *norm1, *norm2;  /* [hidden] RMSNorm gains before attention / before the FFN */
} sr_layer_weights;

typedef struct {
    const void *embed;              /* [vocab][hidden] */
    const void *lm_head;            /* [vocab][hidden]; ignored when tied_lm_head == 1 */
    const void *final_norm;         /* [hidden] */
    const sr_layer_weights *layers; /* HOST array of n_layers entries (of device pointers) */
} sr_weights;

typedef struct {
    int64_t decoded_tokens;   /* tokens appended by sr_decode_step, summed over sequences */
    int64_t prefill_tokens;   /* tokens appended by sr_prefill_chunk (shared prompt counted once per group) */
    int32_t n_live_groups, n_live_seq, seq_len, turn;
    int32_t pages_total, pages_in_use;
    int32_t groups_retired;   /* total over all gates so far */
    int32_t pages_freed;      /* total over all gates so far */
    int32_t cow_page_copies;  /* pages duplicated because a member appended into a shared page */
    int32_t seqs_finished;    /* sequences taken out by sr_finish_sequences */
    int32_t groups_finished;  /* groups that left because their last member finished (not retired by the gate) */
} sr_stats_t;

/*
 * Create a context for n_groups groups of G sequences each and threshold d_L
 * (Eq. 2; resolved to the rational round(d_L*1e6)/1e6).  Allocates the KV pool and all
 * scratch on the current device.  *out is set on success.
 * SR_E_ARG: null pointers, G < 2, unsupported shape/options; SR_E_NOMEM / SR_E_HIP: allocation failed.
 */
int sr_init(sr_ctx **out, const sr_model_shape *shape, int n_groups, int G, double threshold,
            const sr_options *opt);

/* Release everything the context owns.  Synchronises the device.  NULL is allowed. */
void sr_destroy(sr_ctx *ctx);

/*
 * Copy the weights into the library's own packed layout (device -> device, on `stream`)
 * and wait for completion; the caller may free its tensors afterwards.
 */
int sr_load_weights(sr_ctx *ctx, const sr_weights *w, void *stream);

/*
 * Append chunk_len tokens to every live sequence and leave the logits that follow the
 * last of them (Section 2.2: the environment's observation is appended before each action;
 * Appendix C.2: observation tokens are injected, not generated).
 *   shared_per_group = 1: tokens is device int32 [n_live_groups][chunk_len]; the chunk is the
 *       prompt common to the G members of a group; its KV pages are computed once and
 *       shared by the members (copy-on-write).  Only legal while every sequence is empty.
 *   shared_per_group = 0: tokens is device int32 [n_live_seq][chunk_len], one chunk per
 *       sequence; starts a new turn (the next sr_decode_step records the turn's action).
 * SR_E_ARG: bad arguments or max_seq_len exceeded; SR_E_NOMEM: not enough free KV pages
 * (nothing is launched); SR_E_STATE: shared prefill on non-empty sequences, weights not loaded.
 * With no live group the call is a no-op returning SR_OK.
 */
int sr_prefill_chunk(sr_ctx *ctx, const int32_t *tokens, int chunk_len, int shared_per_group,
                     void *stream);

/*
 * One generation step of every live trajectory (Section 2.2: rollout is token-by-token sampling, one
 * model call per environment step and trajectory, and is what dominates the wall-clock; Appendix C.1:
 * the per-step loop over the group's trajectories that the gate interrupts).
 * Decode one token for every live sequence: pick token = forced[r] if forced != NULL, else
 * the library's own choice -- greedy (largest current logit, lowest index on ties) or, with
 * temperature > 0, the sampled token; append it and compute the logits that follow it.
 * out_tokens (device int32 [n_live_seq], may be NULL) always receives the library's own
 * choice, also under forcing.  On the first decode step after a
 * per-sequence prefill the turn's action id (token % action_mod, from the token actually
 * appended) is recorded in the action table.
 * SR_E_STATE before any prefill; SR_E_ARG when max_seq_len would be exceeded; SR_E_NOMEM
 * when a needed KV page cannot be allocated.
 */
int sr_decode_step(sr_ctx *ctx, const int32_t *forced, int32_t *out_tokens, void *stream);

/*
 * Evaluate the gate after turn K = `turn` (1-based count of recorded actions compared):
 * for each live group S_K = sum over the G(G-1)/2 member pairs of the Levenshtein distance
 * between their first K action ids (Section 3.2; all members hold K actions, so
 * d_K = S_K / (C(G,2)*K)), and retire = [d_K < d_L] (Eq. 2, strict) evaluated in integers as
 * S_K < ceil(round(d_L*1e6) * C(G,2) * K / 1e6).
 * out_sums (device int32 [n_live_groups]) and out_retire (device uint8 [n_live_groups]) may
 * be NULL; the mask is also kept inside the context for sr_retire_and_compact.
 * SR_E_ARG: turn < 1 or > max_turns; SR_E_STATE: fewer than `turn` actions recorded.
 */
int sr_gate(sr_ctx *ctx, int turn, int32_t *out_sums, uint8_t *out_retire, void *stream);

/*
 * The cut itself (Section 3.2, paragraph "The gate": when the gate fires, every trajectory of the group
 * that has not ended yet is stopped after step K and the remaining steps are never generated; Appendix
 * C.1: the cut group is skipped by the trainer).
 * Apply the mask of the preceding sr_gate: rows of retired groups are removed from every
 * per-sequence array (order of survivors kept), their KV pages are released (a shared
 * prompt page returns to the pool when its last holder leaves) and the batch shrinks.
 * This call waits for the mask on the host (the one synchronisation per gate turn) and
 * stores the number of surviving groups in *host_n_live_groups (may be NULL).
 * Retiring every group is legal; later prefill/decode calls are then no-ops.
 * SR_E_STATE: no gate since the last compaction.
 */
int sr_retire_and_compact(sr_ctx *ctx, int *host_n_live_groups, void *stream);

/*
 * Take single sequences out of the batch because their trajectory has ended (success or failure
 * reported by the environment) while other members of their group go on (Section 3.2, paragraph
 * "The gate", cuts only the trajectories that have not ended by step K, so some may have; Appendix B
 * defines the fraction that has, tau_K).  host_done: HOST uint8 [n_live_seq], non-zero = finished.  Call
 * between a turn's last sr_decode_step and the next sr_prefill_chunk: the sequence is recorded as
 * finished after `turn` environment steps.  Its private KV pages are freed and its references to
 * the shared prompt pages dropped; its action prefix is kept, because a later sr_gate still
 * compares it with the other members' (a pair is then divided by the longer of the two prefix
 * lengths, Section 3.2, and the member counts towards tau_K).  A group whose last member
 * finishes leaves the batch without being retired.  Rows keep their order; page table and row
 * maps are re-uploaded behind the work already queued.  *host_n_live_seq (may be NULL) receives
 * the number of sequences left.  SR_E_STATE: before the first turn, in the middle of one, or between
 * sr_gate and sr_retire_and_compact (the pending mask is indexed by the groups live at the gate).
 * After this call sr_gate writes to out_sums the plain sum of the pair distances.
 */
int sr_finish_sequences(sr_ctx *ctx, const uint8_t *host_done, int *host_n_live_seq, void *stream);

/*
 * Stand-alone gate over many groups and several prefix lengths (no context needed).
 * actions: device int32 [n_groups][G][stride]; prefix_lens: HOST int [n_lens], each in
 * [1, min(stride, 32)]; sums: device int32 [n_lens][n_groups]; retire: device uint8
 * [n_lens][n_groups] (either may be NULL).  2 <= G <= 16, n_lens <= 8.
 */
int sr_gate_batch(const int32_t *actions, int n_groups, int G, int stride, const int *prefix_lens,
                  int n_lens, double threshold, int32_t *sums, uint8_t *retire, void *stream);

/*
 * sr_gate_batch computed by the other work decomposition -- one workgroup per group, every pair's
 * Levenshtein table advanced one anti-diagonal at a time with the last three anti-diagonals in LDS --
 * for measuring the two side by side.  Same arguments, same results bit for bit (Section 3.2, Eq. 2).
 */
int sr_gate_batch_antidiag(const int32_t *actions, int n_groups, int G, int stride, const int *prefix_lens,
                           int n_lens, double threshold, int32_t *sums, uint8_t *retire, void *stream);

/*
 * Teacher-forced scoring (Appendix C.2).  Appends chunk_len given tokens to every live sequence
 * exactly like sr_prefill_chunk(..., shared_per_group = 0) -- their K/V are computed and the
 * logits at the chunk's last position are kept -- and adds, for every chunk position t whose
 * action_mask entry is non-zero, log softmax(logits at the position before t)[tokens[t]] to the
 * sequence's running log-likelihood  log p(tau) = sum over action-token positions.  A token is scored
 * by the distribution computed from everything before it, so the chunk's first token is scored by the
 * logits the previous prefill / scoring / decode call left and the context must not be empty
 * (SR_E_STATE).  Observation tokens are either passed with mask 0 or, cheaper, appended with
 * sr_prefill_chunk, which computes no LM head for them.
 *
 * tokens: device int32 [n_live_seq][chunk_len]; action_mask: device uint8, same shape, or NULL
 * (every token counts); out_token_logprob: device float [n_live_seq][chunk_len] receiving the
 * per-token values (0 where masked), or NULL.  Arithmetic: bf16 operands, fp32 accumulation and
 * fp32 log-sum-exp per row; the per-sequence sums are kept in double, added in token order.
 * The running sums follow their sequences through sr_retire_and_compact.
 */
int sr_score_chunk(sr_ctx *ctx, const int32_t *tokens, const uint8_t *action_mask, int chunk_len,
                   float *out_token_logprob, void *stream);

/* Copy the running log-likelihoods of the live sequences to dst: device double [n_live_seq]. */
int sr_get_logprob(sr_ctx *ctx, double *dst, void *stream);

/*
 * Policy-gradient loss of Section 2.1:  L = -(1/N) sum_i A_i log p(tau_i)  over the N = n_groups * G
 * trajectories, with the group-relative advantages of Eq. 1 (population standard deviation;
 * every advantage of a group whose rewards are all equal is exactly 0).  No context needed.
 * logprob: device double [n_groups][G]; rewards: device float [n_groups][G]; advantages: device
 * float [n_groups][G] or NULL; group_scratch: device double [n_groups], overwritten; loss: device
 * double [1].  Groups are added in index order, so the result is reproducible.
 */
int sr_grpo_loss(const double *logprob, const float *rewards, int n_groups, int G, double eps,
                 float *advantages, double *group_scratch, double *loss, void *stream);

/*
 * sr_grpo_loss for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without group_scratch,
 * same kernel, same results bit for bit; the per-group shares go to a fixed device array inside the library
 * (SR_GRPO_STATIC_MAX_GROUPS doubles = 512 KiB, held by every GPU the library runs on until the process
 * ends).  The call allocates and frees nothing.  n_groups above the limit: SR_E_LIMIT, nothing is launched.
 * All calls on one GPU share that array: calls that may overlap on one GPU (different streams) race and
 * must be serialised by the caller; nothing of an earlier call's contents is read.
 */
#define SR_GRPO_STATIC_MAX_GROUPS 65536
int sr_grpo_loss_static(const double *logprob, const float *rewards, int n_groups, int G, double eps,
                        float *advantages, double *loss, void *stream);

/*
 * The in-group divergence signals of Appendix B at step K, and the gates of Eq. 2 and of
 * Appendix E (Eq. 3), for groups whose members may have finished early (no context needed).
 *
 * Member i of a group finished after end_step[i] environment steps (any value > stride while
 * it is still running; values below 0 count as 0), so at step K it contributes the prefix
 * a_i[0 : len_i], len_i = min(K, end_step[i]).
 *   d_K            mean over the C(G,2) pairs of the Levenshtein distance of the two prefixes
 *                  divided by the longer of their lengths (Section 3.2); a pair of empty
 *                  prefixes counts 0
 *   lev_scaled     the same sum before the division by C(G,2), exact, in units of
 *                  1 / lcm(1..32) = 1 / 144403552893600
 *   lev_sum        the plain sum over pairs of the Levenshtein distances (S_K when nobody has
 *                  finished early)
 *   bigram_jaccard mean over pairs of 1 - |A n B| / |A u B|, A and B the SETS of consecutive
 *                  action pairs of the two prefixes; two empty sets count as identical (0)
 *   unique_prefix  number of distinct prefixes among the G members (the ratio is this / G)
 *   n_at_step      members whose prefix reaches step K; the next three are taken over them
 *   unique_action  distinct step-K actions a_{i,K}; unique_obs: distinct step-K observation
 *                  ids o_{i,K} (0 if obs is NULL); action_entropy: Shannon entropy of the
 *                  step-K action, natural logarithm
 *   n_done         members that had finished by step K (end_step <= K); tau_K = n_done / G
 *   cut_d          d_K < d_L (Eq. 2, strict), decided in integers with d_L read as
 *                  round(d_L * 1e6) / 1e6;  cut_or: cut_d or tau_K >= tau_H (Eq. 3), tau_H
 *                  read the same way (a tau_H above 1 switches the second clause off)
 * Pair terms are added in the order (0,1), (0,2), ..., (G-2,G-1), so d_K and bigram_jaccard
 * are reproducible bit for bit.
 *
 * actions, obs: device int32 [n_groups][G][stride] (obs may be NULL); end_step: device int32
 * [n_groups][G] or NULL (nobody has finished); prefix_lens: HOST int [n_lens], each in
 * [1, min(stride, 32)]; out: device [n_lens][n_groups].  2 <= G <= 16, n_lens <= 8.
 * SR_E_ARG on anything else.  Asynchronous on `stream`; the caller owns every buffer.
 */
typedef struct {
    double d_K;
    int64_t lev_scaled;
    double bigram_jaccard;
    double action_entropy;
    int32_t unique_prefix, n_at_step, unique_action, unique_obs, n_done;
    int32_t lev_sum;
    uint8_t cut_d, cut_or;
    uint8_t reserved[6];
} sr_signals_t;
int sr_signals_batch(const int32_t *actions, const int32_t *obs, const int32_t *end_step, int n_groups, int G,
                     int stride, const int *prefix_lens, int n_lens, double d_L, double tau_H,
                     sr_signals_t *out, void *stream);

/* Overwrite the action ids of turn `turn` (1-based) for all live sequences:
 * ids is device int32 [n_live_seq].  For action_mod == 0, or for tests. */
int sr_set_actions(sr_ctx *ctx, int turn, const int32_t *ids, void *stream);

/* Copy the action table of the live sequences: dst is device int32 [n_live_seq][max_turns];
 * turns not yet recorded hold -1. */
int sr_get_actions(sr_ctx *ctx, int32_t *dst, void *stream);

/* Copy the current logits: dst is device float [n_live_seq][vocab]. */
int sr_get_logits(sr_ctx *ctx, float *dst, void *stream);

/* Original sequence index (group*G + member at sr_init time) of every live row:
 * host int32 [n_live_seq].  Host-side bookkeeping only; does not touch the stream. */
int sr_get_live_map(sr_ctx *ctx, int32_t *host_orig_seq_ids);

/* Counters (host struct). */
int sr_stats(sr_ctx *ctx, sr_stats_t *host_stats);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of sr_prefill_chunk /
 * sr_decode_step is bracketed by HIP events on the caller's stream (this perturbs the stream
 * slightly; enable it for sampled steps only).  sr_profile_read waits for the stream, adds the
 * elapsed times up per kernel class and clears the record.  Classes are numbered by
 * sr_kernel_class; `out` is a HOST array of SR_KC_COUNT entries.
 */
typedef enum {
    SR_KC_NORM = 0,        /* residual add + RMSNorm (+ embedding gather) */
    SR_KC_GEMM_QKV,
    SR_KC_QKV_POST,        /* split-K sum + bias + RoPE + KV page write */
    SR_KC_ATTN_DECODE,     /* decode attention: shared-prompt phase and private phase in one launch */
    SR_KC_ATTN_PREFILL,
    SR_KC_ATTN_MERGE,
    SR_KC_GEMM_O,
    SR_KC_GEMM_GATE_UP,    /* with the SwiGLU epilogue */
    SR_KC_GEMM_DOWN,
    SR_KC_GEMM_LM_HEAD,
    SR_KC_ARGMAX,
    SR_KC_COUNT
} sr_kernel_class;

typedef struct {
    int64_t launches;
    double total_ms;
} sr_kernel_time;

int sr_profile(sr_ctx *ctx, int enable);
int sr_profile_read(sr_ctx *ctx, sr_kernel_time *host_out /* [SR_KC_COUNT] */, void *stream);

/*
 * Measured ceilings of the chip, for the roofline report next to the published peaks (HBM 8 TB/s, dense
 * bf16 matrix cores 2.5 PFLOP/s).  Both calls launch probe kernels on `stream`, time `iters` launches with
 * HIP events, wait for them and write the rate to a HOST double.  They are not part of the method.
 *   sr_probe_hbm: src (device, `bytes` long; use well over 256 MiB so that no cache holds it) is streamed by
 *     4096 wavefronts with 16-byte loads -- mode 0 with the non-temporal hint of the weight-streaming kernels,
 *     mode 1 with default loads, mode 2 copied to dst (device, `bytes` long; read + written bytes are counted).
 *     For modes 0 and 1 dst must point at >= 16 device bytes (never written in practice).
 *   sr_probe_mfma_bf16: register-resident 32x32x16 bf16 matrix-core loop on 1024 workgroups; scratch is
 *     device memory of at least 1 MiB that receives one float per thread.
 */
int sr_probe_hbm(const void *src, void *dst, size_t bytes, int mode, int iters, void *stream, double *host_GBs);
int sr_probe_mfma_bf16(void *scratch, size_t scratch_bytes, int iters, void *stream, double *host_TFLOPs);

/*
 * The matrix-core loop with operand-sized loads beside it, for telling what the operand traffic of a tiled GEMM leaves
 * of the matrix pipe: 256 workgroups of eight wavefronts; every wavefront alternates sixteen register-resident
 * 32x32x16 bf16 MFMAs with loads_per_16 (2, 4 or 8; 0 with path 0) wavefront-wide loads of 16 bytes per lane from buf,
 * into registers (path 1) or straight into LDS (path 2); lds_reads != 0 adds twelve 16-byte LDS reads per sixteen MFMAs
 * (paths 0 and 2).  A 256 x 256 x 32 GEMM step on eight computing wavefronts corresponds to loads_per_16 = 4.
 * buf: device memory, buf_bytes a power of two >= 64 KiB (small = L2 resident; read only).  scratch: device memory of
 * at least 512 KiB that receives one float per thread.  Waits for the stream; writes the matrix rate and the rate of
 * the loads to HOST doubles (host_load_GBs may be null).  SR_E_ARG for any other combination.
 */
int sr_probe_mfma_under_loads(const void *buf, size_t buf_bytes, void *scratch, size_t scratch_bytes, int path,
                              int loads_per_16, int lds_reads, int iters, void *stream, double *host_TFLOPs,
                              double *host_load_GBs);

/*
 * One layer's decode attention launch at the 7B attention shape (28 query / 4 kv heads of 128, 64-token pages) on
 * synthetic pages, for studying its phases apart: phases = 1 the shared-prompt phase alone (one unit per group, the
 * members' query rows batched over each prompt block), 2 the private phase alone (one unit per sequence, priv_splits
 * splits of priv_tokens tokens), 3 both in one launch as sr_decode_step runs them; adding 4 puts the launch that merges
 * the partial results behind each attention launch (the duration is then that of the pair).  hot != 0: every page-table entry
 * names one of a few pages, so all K/V loads are cache hits.  Allocates and frees its own buffers, waits for the
 * stream, and writes the mean launch duration in microseconds and the K/V bytes one launch has to read to HOST doubles.
 */
int sr_probe_decode_attention(int n_groups, int G, int shared_tokens, int priv_tokens, int priv_splits, int phases,
                              int hot, int iters, void *stream, double *host_us, double *host_kv_bytes);

/* Text for a status code; for SR_E_HIP the text of the last HIP error seen by this thread. */
const char *sr_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SR_H */
