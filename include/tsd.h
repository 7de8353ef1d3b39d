/*
 * tsd.h -- C ABI of libtsd: batched Gaussian speculative decoding rounds for continuous
 * patch-autoregressive time-series transformers on AMD MI355X (gfx950).
 *
 * The method (arXiv 2511.18191): a cheap draft model proposes K future patches, the target
 * model scores all K+1 prefix boundaries in ONE causal pass, each proposal passes a log-domain
 * Gaussian likelihood-ratio test, the first rejection is replaced by the target's own mean, a
 * bonus patch is committed on full acceptance, and the round ends.  This library runs that
 * round for a whole batch of independent series with per-series ragged accepted lengths, over
 * a paged per-series KV cache, entirely in hand-written HIP kernels.
 *
 * Conventions
 *   - Every function returns TSD_OK (0) or a negative TSD_E_* code; nothing throws or aborts.
 *     Arguments are validated on the host before anything is launched.  tsd_last_error()
 *     returns a human-readable message for the most recent failure on that handle (or, with a
 *     NULL handle, for the most recent failure of a call that had no handle).
 *   - Pointers named *_dev are DEVICE pointers, *_host are HOST pointers.  The caller owns all
 *     device memory (arena, weight blobs, I/O buffers); the library owns only the opaque
 *     handle and never frees or allocates device memory.  Each handle also holds 64 bytes of
 *     pinned host memory (allocated by tsd_create, freed by tsd_destroy): the words through
 *     which the active-series counts reach the host (see tsd_num_active).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All calls are
 *     asynchronous on that stream except where stated.  Calls on one handle must be issued
 *     from one thread at a time and on one stream at a time.
 *   - All arrays are dense row-major.  Patches live in NORMALISED space (per-series mean/std
 *     of the context, frozen at prefill: Sec. "Single-Pass Verification"); only
 *     tsd_get_forecast() de-normalises.
 *   - dtype TSD_F32: weights, activations and KV in fp32.  dtype TSD_BF16: weights, KV and
 *     GEMM operands in bf16, accumulation / norms / softmax / RoPE / residual stream / model
 *     outputs / acceptance in fp32.
 *
 * Model evaluated (the paper fixes a decoder-only causal transformer with a point head and
 * the layer/width/head/FFN counts; the rest is this library's documented choice):
 *   e_j = patch_j W_e; per layer: a = RMSNorm(x; g1, eps 1e-6); q,k,v = a W_q, a W_k, a W_v;
 *   half-split RoPE (base 10000, position = absolute token index) on q,k; causal softmax
 *   attention with scale 1/sqrt(head_dim); x += attn W_o; b = RMSNorm(x; g2);
 *   dense: x += GELU_tanh(b W_1) W_2;  routed: softmax router over n_experts, top_k by
 *   probability (ties to the lower index), gates renormalised to sum 1, x += sum gate_e FFN_e(b);
 *   mu_j = RMSNorm(x_j; g_f) W_h = predicted mean of patch j+1.  No biases.
 */
#ifndef TSD_H
#define TSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TSD_OK 0
#define TSD_E_INVALID_ARG (-1)  /* NULL pointer, bad size, unsupported shape               */
#define TSD_E_BAD_STATE (-2)    /* call made out of order (e.g. round before prefill)      */
#define TSD_E_OUT_OF_RANGE (-3) /* batch / tokens exceed what the handle was created for   */
#define TSD_E_HIP (-4)          /* a HIP runtime call failed; see tsd_last_error()         */

#define TSD_F32 0
#define TSD_BF16 1

#define TSD_TARGET 0
#define TSD_DRAFT 1

/* flags */
#define TSD_FLAG_SCRAMBLE_PAGES 1u /* assign physical KV pages by a pseudo-random permutation */
#define TSD_FLAG_NO_TEMPERING 2u   /* ablation: use d * ell (drop the 1/d scaling of Eq. 5)    */
#define TSD_FLAG_NO_GRAPH 4u       /* launch kernels one by one instead of replaying HIP graphs */
#define TSD_FLAG_NO_COMPACT 8u     /* always run passes over the whole batch (see tsd_num_active) */
#define TSD_FLAG_NO_SKINNY 16u     /* never use the <= 32-row weight-streaming GEMM                */
#define TSD_FLAG_SAMPLE_PROPOSALS 32u /* ablation: x_i = mu_q^(i) + sigma_q eps instead of the mean */
#define TSD_FLAG_NAIVE_VERIFY 64u  /* ablation: one target pass per prefix instead of one causal pass */
#define TSD_FLAG_THRESHOLD_RULE 128u /* variant: accept iff ||x_i - mu_p^(i)||_d^2 <= sigma_p^2, no draw */
#define TSD_FLAG_BATCH_SYNC 256u   /* variant: every series keeps the batch's smallest accepted count */
#define TSD_FLAG_NO_PINNED_COUNTS 512u /* tsd_num_active copies the counts back and waits on the stream */
#define TSD_FLAG_NO_FUSED_DRAFT 1024u /* always run the draft phase kernel by kernel                       */
#define TSD_FLAG_FUSED_DRAFT 2048u /* run the draft phase as one launch wherever that kernel is supported */
#define TSD_FLAG_NO_WIDE_GEMM 4096u /* never use the wide-tile direct-to-LDS GEMM kernels (same bits, for A/B timing) */

typedef struct tsd_ctx tsd_ctx; /* opaque */

typedef struct {
  int32_t n_layers, d_model, n_heads, d_ff;
  int32_t n_experts; /* 0 = dense FFN, else 2..16 routed experts          */
  int32_t top_k;     /* experts per token when n_experts > 0, 1..min(4, E) */
} tsd_model_cfg;

typedef struct {
  tsd_model_cfg target, draft;
  int32_t patch;       /* P: steps per patch (= acceptance dimension d, one channel per series) */
  int32_t K;           /* proposals per round, 1..16                                            */
  int32_t max_batch;   /* largest B accepted by tsd_prefill                                     */
  int32_t max_tokens;  /* largest N + ceil(H/P) + K accepted by tsd_prefill                     */
  int32_t dtype;       /* TSD_F32 | TSD_BF16                                                    */
  int32_t page_tokens; /* tokens per KV page (power of two, 1..64)                              */
  float sigma_p;       /* acceptance temperature of the target surrogate (Eq. 4)                */
  float sigma_q;       /* ... of the draft surrogate; equal to sigma_p in the deployed scheme   */
  float fallback_r;    /* fallback noise r in [0, sigma_p]; 0 = target-mean fallback (deployed) */
  uint32_t flags;
  uint64_t seed;       /* Philox key = (low 32 bits, high 32 bits)                              */
} tsd_config;

typedef struct {
  int64_t rounds;     /* series-rounds executed (one per active series per round)            */
  int64_t tested;     /* proposals that met the acceptance test                              */
  int64_t accepted;   /* proposals accepted by the test (before any forced length)           */
  int64_t committed;  /* patches committed (after truncation at T)                           */
  int64_t near_ties;  /* tested proposals with |min(0, ell) - log u| < 1e-4                   */
} tsd_stats;

/* Bytes of device memory tsd_create needs for `cfg` (weights in internal layout, rotary
 * tables, both paged KV pools, page table, per-series state, activation workspace).
 * One size for one arena: the KV pools and the scratch share an allocation the caller makes
 * once, instead of a KV size and a scratch size for two; the library carves it (256-byte
 * aligned parts) and never allocates device memory itself.
 * Host-only; never touches the GPU. */
int tsd_workspace_bytes(const tsd_config* cfg, size_t* bytes_host);

/* Number of float32 elements of one model's weight blob (`which` = TSD_TARGET | TSD_DRAFT).
 * Blob order: W_e [P,D]; per layer: g1 [D], W_q, W_k, W_v, W_o [D,D], g2 [D], then
 * dense: W_1 [D,F], W_2 [F,D]; routed: W_r [D,E], then per expert W_1 [D,F], W_2 [F,D];
 * finally g_f [D], W_h [D,P].  Matrices are stored as used in y = x W (row-major [in,out]).
 * Host-only. */
int tsd_weights_count(const tsd_config* cfg, int which, size_t* n_floats_host);

/* Create a handle over caller-owned device memory `arena_dev` (256-byte aligned, at least
 * tsd_workspace_bytes).  The arena must outlive the handle.  Fills the rotary tables
 * (synchronous host-to-device copies). */
int tsd_create(const tsd_config* cfg, void* arena_dev, size_t arena_bytes, tsd_ctx** out);

/* Release the handle (host memory only).  Synchronises the device first. */
int tsd_destroy(tsd_ctx* ctx);

/* Convert one model's float32 blob (device memory, order above) into the internal layout
 * (transposed, RMSNorm gains folded into the following matrix, rounded to bf16 when
 * dtype = TSD_BF16).  The blob may be freed once the stream has passed this call. */
int tsd_load_weights(tsd_ctx* ctx, int which, const float* blob_dev, size_t n_floats, void* stream);

/* Start a forecast for B series.  series_dev: [B, n_ctx_patches * P] raw context steps.
 * Computes the frozen per-series statistics (mean, sqrt(population variance + 1e-5)),
 * normalises, runs target and draft over context patches 0..N-2 to fill both KV caches, and
 * keeps patch N-1 as the pending (not yet ingested) token.  Requires n_ctx_patches >= 2,
 * B <= max_batch, n_ctx_patches + ceil(horizon_steps / P) + K <= max_tokens. */
int tsd_prefill(tsd_ctx* ctx, const float* series_dev, int32_t B, int32_t n_ctx_patches, int32_t horizon_steps,
                void* stream);

/* Continuous batching (the desynchronisation remedy the paper points to: a batch is as slow as
 * its slowest series, so finished slots are handed to new series instead of idling).  Replaces the
 * series in the `n` slots slots_host[0..n-1] (host array, distinct indices in 0..B-1) by new ones:
 * series_dev is [n, n_ctx_patches * P] raw context steps with the n_ctx_patches and horizon of the
 * running tsd_prefill.  Per slot: frozen statistics, normalisation, both models' KV entries of the
 * context (the slot's pages are reused), cache length, committed count and the active flag start
 * over; the slot's round counter keeps running, so the acceptance draws of successive series in
 * one slot never repeat, and its statistics keep accumulating.  A slot that is still decoding
 * loses its forecast.  Read finished forecasts (tsd_get_forecast) before refilling their slots,
 * and call tsd_num_active afterwards.  Synchronises `stream` on entry. */
int tsd_refill(tsd_ctx* ctx, const int32_t* slots_host, int32_t n, const float* series_dev, void* stream);

/* Rewind to the state right after tsd_prefill (KV entries of the context are kept, everything
 * committed since is dropped, statistics zeroed).  Lets one prefill serve several decodes. */
int tsd_reset_decode(tsd_ctx* ctx, void* stream);

/* Algorithm "One speculative round", first loop: K sequential draft passes; proposal i is the
 * draft's mean given the history and proposals 1..i-1 (mean-propagating scheme, x_i = mu_q^(i)).
 * With TSD_FLAG_SAMPLE_PROPOSALS (Sec. "Fallback Correction and Sampled Variants", an ablation
 * knob) proposal i is the draw x_i = mu_q^(i) + sigma_q eps_i, which the next draft step and the
 * target then consume.  eps: element e of the patch of (series b, that series' round r, position
 * i) comes from Philox4x32-10 with counter (b, r, i, stream * 2^16 + e / 4), stream = 1 for
 * proposals and 2 for the fallback patch: the block's four words give lattice uniforms u0..u3
 * (as for the acceptance uniform) and the Box-Muller pairs sqrt(-2 ln u0) (cos, sin)(2 pi u1),
 * sqrt(-2 ln u2) (cos, sin)(2 pi u3); element e takes number e mod 4.
 * Fills the internal X [B,K,P] (and mu_q [B,K,P] when sampling).  Once tsd_num_active has
 * reported that no active series needs K more patches, only min(K, largest need) steps run and
 * the later rows of X keep stale values (no series tests them).
 * A dense bf16 draft with head_dim 64 whose 16-row working set fits one compute unit's LDS can run
 * the whole phase as ONE launch (a workgroup keeps a few series through all steps and layers,
 * streaming the draft weights once per step); the per-row arithmetic is that of the kernel-by-kernel
 * path up to the summation order inside the products (sampled proposals are drawn inside it from
 * the same counters).  It is the default where it was measured to
 * win (draft weights of at most 4 MiB, widths in multiples of 256, more than 32 rows per pass and
 * max_batch <= 512);
 * TSD_FLAG_FUSED_DRAFT selects it wherever it is supported, TSD_FLAG_NO_FUSED_DRAFT never. */
int tsd_draft_propose(tsd_ctx* ctx, void* stream);

/* Single-pass verification (Sec. "Single-Pass Verification"): one causal target pass over the
 * pending token and x_1..x_K against the paged KV cache; the output at token j is the target
 * mean at prefix boundary j+1.  Fills the internal mu_p [B,K+1,P].
 * With TSD_FLAG_NAIVE_VERIFY (the component ablation's "w/o single-pass verification") each of
 * the K+1 prefixes is re-encoded by its own pass against the cached context and only its last
 * boundary is read: same mu_p up to rounding, (K+1)(K+2)/2 target tokens per round. */
int tsd_target_verify(tsd_ctx* ctx, void* stream);

/* Acceptance (Eq. 5 / Eq. 6), correction, commit and KV rollback for every active series:
 *   ell_i = -||x_i - mu_p^(i)||_d^2 / (2 sigma_p^2) + ||x_i - mu_q^(i)||_d^2 / (2 sigma_q^2)
 *           + (1/2) log(sigma_q^2 / sigma_p^2),     ||u||_d^2 = ||u||^2 / P;
 *   u_i = Philox4x32-10(counter = (series, round of that series, i, 0), key = seed), word 0,
 *         u = ((w >> 9) + 0.5) * 2^-23;   accept iff log u_i <= min(0, ell_i), left to right;
 *   a series with r = T - committed patches left (T = ceil(H/P)) tests only positions
 *   1..K_b, K_b = min(K, r): nothing is proposed for patches that could never be committed;
 *   n = number of leading accepts; commit x_1..x_n then mu_p^(n+1) (fallback if n < K_b, bonus
 *   if n = K_b), truncated at T patches (which drops a bonus patch at T + 1); both KV caches keep exactly the entries of
 *   the committed history; mu_p^(n+1) becomes the pending token; a series with T patches
 *   becomes inactive.  With fallback_r = r > 0 the corrected / bonus patch is the draw
 *   mu_p^(n+1) + r eps (stream 2, position n+1; Sec. "Bonus Patch on Full Acceptance").
 * With TSD_FLAG_THRESHOLD_RULE (Table "TiRex configuration", row "Acceptance draw") the test is
 * deterministic: position i passes iff ||x_i - mu_p^(i)||_d^2 <= sigma_p^2 (per-dimension scales:
 * the scaled Mahalanobis distance is at most 1).  It is evaluated and recorded in the log form
 * ell_i = -||x_i - mu_p^(i)||_d^2 / (2 sigma_p^2) against the constant log u_i = -1/2; no uniform
 * is drawn and the draft-side terms of Eq. 5 are not used.
 * With TSD_FLAG_BATCH_SYNC (same row: the batch is kept in step) the series taking part in the round
 * first find their own counts, then all of them keep the smallest one: each commits its first
 * n_min proposals and its own mu_p^(n_min + 1), so series that start together stay at the same
 * length.  The statistics' tested / accepted and the n_acc tap keep each series' own test;
 * committed follows n_min.  Costs two more small launches per round.
 * forced_len_dev (nullable): int32 [B]; entry b in 0..K overrides n for series b after the test
 * has been evaluated and recorded (used to keep two implementations in lock-step); -1 = free.
 * Under TSD_FLAG_BATCH_SYNC the overridden value is the series' own count that enters the minimum. */
int tsd_accept_commit(tsd_ctx* ctx, const int32_t* forced_len_dev, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it) and that run their own models: the acceptance / correction / commit step of ONE
 * round (the rule of tsd_accept_commit, same kernel) on caller tensors, without a handle or an arena.  The
 * state the kernel keeps (per-series round counter, committed count, active flag, pending / previous token,
 * counters, the synchronised round's minimum) lives in a fixed device array inside the library, about 2.8 MB,
 * held on every GPU the library has run this call on until the process ends; the call allocates nothing and
 * frees nothing.  Limits: B <= 4096, K <= 16, B * P <= 262144; larger sizes return TSD_E_OUT_OF_RANGE.
 *   inputs (device): X, mu_q [B,K,P]; mu_p [B,K+1,P]; round_dev int32 [B] (nullable = all 0): the second word
 *     of each series' Philox counter, as the handle keeps it per series.
 *   sigma_p, sigma_q, fallback_r, seed: as in tsd_config.  flags: TSD_FLAG_NO_TEMPERING, TSD_FLAG_THRESHOLD_RULE
 *     and TSD_FLAG_BATCH_SYNC apply; any other bit is an error.
 *   outputs (device): n_acc int32 [B]: leading accepts found by each series' own test; commit [B,K+1,P]: rows
 *     0..n-1 = x_1..x_n and row n = the corrected (n < K) or bonus (n = K) patch, n = n_acc or, synchronised, the
 *     batch's smallest; later rows are left untouched; ell, logu [B,K] (nullable): the statistics and log draws,
 *     NaN where a position was not tested.
 * Every call on a GPU shares that GPU's array and overwrites the previous call's state (nothing carries over:
 * the state is set up afresh by a small kernel at the start of every call); calls that overlap on one GPU,
 * on different streams or from different threads, race.  Asynchronous on `stream`. */
int tsd_accept_commit_static(const float* X_dev, const float* mu_q_dev, const float* mu_p_dev, const int32_t* round_dev,
                             int32_t B, int32_t K, int32_t P, float sigma_p, float sigma_q, float fallback_r,
                             uint64_t seed, uint32_t flags, int32_t* n_acc_dev, float* commit_dev, float* ell_dev,
                             float* logu_dev, void* stream);

/* tsd_draft_propose; tsd_target_verify; tsd_accept_commit(NULL).  On a non-NULL stream that is not
 * being captured by the caller, the launch sequence is captured into a HIP graph on first use and
 * replayed afterwards (same for tsd_target_step); TSD_FLAG_NO_GRAPH switches that off.  Graphs are
 * kept per number of positions the round runs and per size class of the active list (launches
 * sized for 1/32 .. 32/32 of the batch); the class is chosen from the last length the host has
 * seen, looked up without waiting, and every launch is capped by the device-side length. */
int tsd_round(tsd_ctx* ctx, void* stream);

/* Rounds until no series needs patches any more (or max_rounds rounds have run): the loop
 *   do { tsd_round; tsd_num_active; } while (active > 0)
 * kept inside the library, so that nothing but the count's delivery stands between two rounds.
 * A round commits at most K + 1 patches per series, so while the neediest series is known to need
 * more than that, the next round is enqueued without waiting for the count (only for handles whose
 * passes follow the device-side count; routed models size their passes from every count).  Results are those of
 * the written-out loop, bit for bit.  rounds_host (nullable) receives the number of rounds run,
 * active_host (nullable) the number of series still active at the end.  Synchronises `stream`
 * like tsd_num_active. */
int tsd_run_rounds(tsd_ctx* ctx, int32_t max_rounds, int32_t* rounds_host, int32_t* active_host, void* stream);

/* Target-only autoregressive baseline (Eq. 1) from the same kernels: one target pass over the
 * pending token, whose output is committed for every active series. */
int tsd_target_step(tsd_ctx* ctx, void* stream);

/* Number of series that still need patches.  Synchronises `stream`.  Passes cover only the series
 * on the active list, which the last kernel of every round rebuilds on the device together with
 * its length; this call brings the length to the host.  Launches issued before the next call are
 * sized from the length the host knows (an older, larger one at worst) and capped by the
 * device-side one, so a series that finishes in between costs at most workgroups that leave at
 * once, never a second visit.  Handles whose passes are sized on the host (routed models) keep
 * reading the list as of this call until the next one.
 * Results are identical, to the bit, with or without it (every kernel a shrinking pass may be
 * handed sums in the same order); finished series simply stop costing work.
 * The counts reach the host through a few pinned host words that the compaction kernel writes
 * itself (tsd_round already ends with that kernel), so this call normally launches nothing and
 * waits for nothing but those words; it falls back to a copy and a stream wait when pinned
 * memory could not be allocated at tsd_create. */
int tsd_num_active(tsd_ctx* ctx, int32_t* out_host, void* stream);

/* De-normalised forecast, out_dev: [B, horizon_steps] (first H steps of the committed patches;
 * positions not yet committed are written as 0). */
int tsd_get_forecast(tsd_ctx* ctx, float* out_dev, void* stream);

/* Parity taps: copies of the last round's tensors.  Any pointer may be NULL.
 * X, mu_q: [B,K,P]; mu_p: [B,K+1,P]; n_acc: int32 [B] accepted count found by the test (-1 for
 * series that were inactive when the round ran; rows of series no longer listed keep old values); ell, logu: [B,K] (NaN where a position was not tested). */
int tsd_get_round_io(tsd_ctx* ctx, float* X_dev, float* mu_q_dev, float* mu_p_dev, int32_t* n_acc_dev,
                     float* ell_dev, float* logu_dev, void* stream);

/* Replace the round tensors consumed by the next tsd_accept_commit (kernel-level parity: feed
 * another implementation's X, mu_q, mu_p).  All three required, shapes as above. */
int tsd_set_round_io(tsd_ctx* ctx, const float* X_dev, const float* mu_q_dev, const float* mu_p_dev, void* stream);

/* Parity tap of the routed FFN: while ids_dev is installed, every pass through model `which` also files the
 * experts its router chose under ids_dev[layer][series][absolute token position][choice] (int32, choice 0 = the
 * most probable; series = index in the batch; entries of positions no pass has visited keep what the caller put
 * there).  A top-k choice is discrete: another implementation that is to be compared at a floating-point
 * tolerance has to be evaluated with the same choices wherever its own differ only by rounding.  ids_dev: caller-
 * owned device memory of n_ints >= n_layers * max_batch * max_tokens * top_k entries, valid until the tap is
 * removed (ids_dev = NULL) or the handle destroyed.  Costs one small launch per layer while installed. */
int tsd_set_route_tap(tsd_ctx* ctx, int which, int32_t* ids_dev, size_t n_ints);

/* Per-series state: len int32 [B] (tokens held by the target cache = position of the pending
 * token), committed int32 [B], pending float [B,P].  Any pointer may be NULL. */
int tsd_get_state(tsd_ctx* ctx, int32_t* len_dev, int32_t* committed_dev, float* pending_dev, void* stream);

/* Aggregate counters since prefill / reset.  Synchronises `stream`. */
int tsd_get_stats(tsd_ctx* ctx, tsd_stats* out_host, void* stream);

/* The same five counters per series: out_dev int64 [B,5] in the field order of tsd_stats.  A
 * series' accepted / tested is one [0,1]-valued, independent per-history term of the plug-in
 * acceptance estimate (Proposition "Unbiased plug-in estimator", Theorem "Hoeffding
 * concentration"). */
int tsd_get_series_stats(tsd_ctx* ctx, int64_t* out_dev, void* stream);

/* alpha in (0, 1]: every tested position is accepted with this constant probability instead of
 * min(1, e^ell) (block-length law under an i.i.d. rate, Eq. 7).  alpha < 0 restores the rule. */
int tsd_set_accept_override(tsd_ctx* ctx, float alpha);

/* Change the number of proposals per round to K in 1..(K given to tsd_create), between rounds
 * (Proposition "Marginal-gain condition for K": the block size is chosen from the measured
 * acceptance and cost ratios, which are known only after some rounds have run).  All state a
 * round depends on (cache lengths, pending token, counters) is independent of K; the round
 * tensors are re-laid out for the new K, so tensors injected with tsd_set_round_io are dropped. */
int tsd_set_block_size(tsd_ctx* ctx, int32_t K);

/* Change the acceptance temperatures (temperature sweeps without re-creating the handle).
 * Returns to the isotropic surrogate if tsd_set_sigma_diag was in effect. */
int tsd_set_sigma(tsd_ctx* ctx, float sigma_p, float sigma_q);

/* Diagonal-covariance surrogate (Remark "General covariances"): sigma_p_dev, sigma_q_dev are
 * float32 [P] per-dimension scales on the device (copied; both required, all positive).  The
 * statistic becomes
 *   ell_i = -(1/2P) sum_e (x - mu_p)_e^2 / s_p[e]^2 + (1/2P) sum_e (x - mu_q)_e^2 / s_q[e]^2
 *           + (1/2P) sum_e log(s_q[e]^2 / s_p[e]^2),
 * and sampled proposals draw x_i = mu_q^(i) + s_q * eps element-wise.  Synchronises `stream`
 * (the scales are validated and the inverse variances and the log-det term formed on the host). */
int tsd_set_sigma_diag(tsd_ctx* ctx, const float* sigma_p_dev, const float* sigma_q_dev, void* stream);

/* Measurement tap (not part of the method): time every launch of one kernel family with HIP
 * events recorded on the launching stream.  kernel_class: TSD_K_*; while a class is selected,
 * tsd_round / tsd_target_step launch kernel by kernel (no graph replay).  tsd_profile_end waits
 * for the stream, returns the number of launches, their summed duration in milliseconds and their
 * summed algorithmic work (GEMM families: 2*M*N*K flops; TSD_K_ATTN: bytes of the K and V rows
 * each (series, head) must read, counted with the shortest possible history N-1, plus q and
 * output rows; TSD_K_ACCEPT: bytes of X, mu_p read and the committed patch written; TSD_K_ROUTE:
 * bytes of the rows read and written; the grouped expert GEMMs count under TSD_K_GELU and
 * TSD_K_RESID), and switches the tap off. */
#define TSD_K_EMBED 0  /* patch embedding GEMM                          */
#define TSD_K_QKV 1    /* RMSNorm + QKV GEMM + RoPE + KV-cache write    */
#define TSD_K_ATTN 2   /* paged causal attention                        */
#define TSD_K_RESID 3  /* attention-output and FFN-down GEMMs (+residual) */
#define TSD_K_GELU 4   /* RMSNorm + FFN-up GEMM + GELU                  */
#define TSD_K_HEAD 5   /* RMSNorm + output-head GEMM                    */
#define TSD_K_ACCEPT 6 /* acceptance + commit + rollback                */
#define TSD_K_ROUTE 7  /* routed FFN: router, expert sort, gated combine (bytes) */
#define TSD_K_DRAFT 8  /* the draft phase as one launch (flops of the passes it replaces) */
#define TSD_K_COUNT 9  /* as a kernel_class: every family at once */
int tsd_profile_begin(tsd_ctx* ctx, int kernel_class);
int tsd_profile_end(tsd_ctx* ctx, int64_t* launches_host, double* ms_host, double* work_host, void* stream);

/* The launches of the measurement that the last tsd_profile_end closed, one record each, in launch order:
 * family, model (TSD_TARGET / TSD_DRAFT, -1 for the acceptance kernel), and for the GEMM families the kernel the
 * launcher picked (`tile`: 128 or 64 = tile size of the tiled kernel, 464 = 64 x 64 tiles with K split over four
 * wavefront groups, 16 = the skinny weight-streaming kernel) and the product's shape as launched (rows M as
 * sized on the host: a replayed or device-capped launch may run fewer); attention: M = query rows, N = model
 * width; duration between the two events in milliseconds; algorithmic work as summed by tsd_profile_end.
 * out_host: max_records entries; *n_host receives the number of launches recorded (which may exceed
 * max_records; only the first max_records are stored).  Host-only. */
typedef struct {
  int32_t kernel_class, model, tile, M, N, K;
  float ms;
  double work;
} tsd_launch_rec;
int tsd_profile_launches(tsd_ctx* ctx, tsd_launch_rec* out_host, int32_t max_records, int32_t* n_host);

/* Measurement tap: one product through the same tiled kernel, tile selection and tile order the
 * transformer passes use.  dtype TSD_BF16: A and Wt are bf16; TSD_F32: fp32.  variant 0:
 * C[M,N] = A[M,K] * Wt[N,K]^T (fp32 result); variant 1: the same with each row of the product
 * scaled by rsqrt(mean(A_row^2) + 1e-6) (the fused RMSNorm); variant 2: C += A * Wt^T (the
 * residual epilogue); variant 3 (bf16 only): C = GELU_tanh(RMSNorm-scaled product), stored as bf16 [M,N]: the
 * FFN-up product exactly as the passes run it; variant + 8: the same without the wide-tile kernels.  K must be a
 * multiple of 8, N of 4.  No handle needed. */
int tsd_bench_gemm(int dtype, int variant, int M, int N, int K, const void* A_dev, const void* Wt_dev, void* C_dev,
                   void* stream);

/* Measurement tap: a plain copy kernel (dst[i] = src[i], 16 bytes per lane) of `bytes` bytes
 * (a multiple of 16).  Its known traffic calibrates the profiler's memory counters. */
int tsd_bench_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

/* Measurement tap: `blocks` workgroups of 256 lanes, every wavefront issuing `iters` rounds of four
 * independent v_mfma_f32_32x32x16_bf16 chains on register operands (no memory traffic inside the
 * loop): 2 * 32 * 32 * 16 * 4 * iters flop per wavefront.  The rate it reaches is the matrix-core
 * ceiling this library's GEMM instruction can be priced against on the machine at hand, next to the
 * published peak.  sink_dev: float [blocks * 256], written once at the end (keeps the chains live). */
int tsd_bench_mfma(int32_t blocks, int32_t iters, float* sink_dev, void* stream);

/* Measurement tap of the one-launch draft phase: runs tsd_draft_propose once with workgroup 0 noting the
 * 100 MHz wall clock (s_memrealtime) after every one of its stage barriers, and returns the stamps in
 * order: 2 of the set-up, then per draft step: positions, patch embedding, per layer (QKV, attention,
 * attention output, FFN up, FFN down), head -- 2 + steps * (3 + 5 * layers) values; consecutive
 * differences are stage durations in units of 10 ns.  ticks_host: host array of max_ticks entries;
 * *n_host receives the number of stamps taken (at most 512; only the first max_ticks are stored).
 * The round tensors are left as after tsd_draft_propose.  Synchronises the stream.
 * TSD_E_BAD_STATE if the handle runs the draft phase kernel by kernel. */
int tsd_trace_draft(tsd_ctx* ctx, int64_t* ticks_host, int32_t max_ticks, int32_t* n_host, void* stream);

const char* tsd_last_error(tsd_ctx* ctx);

/* ABI version of this header (bumped on incompatible change). */
int tsd_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TSD_H */
