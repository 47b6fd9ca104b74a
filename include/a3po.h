/*
 * a3po.h - C ABI of the MI355X (gfx950) library for the per-token policy-probability
 * path of A-3PO training (arXiv 2512.06547): vocabulary-wide log-softmax + chosen-token
 * gather, staleness-aware log-linear proximal interpolation, decoupled clipped surrogate
 * with masked token mean, and the gradient written back to the logits.
 *
 * Conventions for every entry point
 *  - Pointers are DEVICE pointers owned by the caller unless marked "host".  The
 *    library never allocates, frees or synchronises; all work is enqueued on `stream`
 *    (a hipStream_t passed as void*, NULL = the default stream) and the call returns
 *    as soon as the launches are queued.  Outputs are valid once the stream reaches them.
 *  - Return value: A3PO_OK (0) or a negative A3PO_E_* code for anything the host can
 *    detect (null pointer, bad size, unknown dtype, misaligned pointer, workspace too
 *    small, launch failure).  Nothing throws or aborts.  T == 0 is success.
 *  - Data-dependent problems cannot be returned synchronously; they are counted in
 *    a3po_stats (chosen id outside [0,V) => the token is treated as masked; negative
 *    staleness => alpha = 1).
 *  - No state is kept between calls: they are re-entrant and may be issued from several host threads
 *    on different streams, as long as they do not share output buffers or a workspace.  (The set-ups
 *    that happen once per device are thread-safe: the LDS limit of the kernels that use more than 64 KiB, and the address of the array that
 *    a3po_loss_fwd_bwd_noalloc uses in place of a workspace.)
 *  - Logits are row-major [T, V] with a row stride of `ld` elements (ld >= V), float32
 *    or bfloat16.  Row t pairs with chosen[t]; any next-token shift is the caller's.
 *    Base pointers of logits / dlogits must be aligned to their element size.  Rows whose base
 *    and byte stride are multiples of 16 take the vectorised kernels: each row is read once and written
 *    once when it fits the registers (V <= 163,840 bfloat16 / 81,920 float32); a longer row stays on chip as
 *    far as registers and LDS hold it (448 KiB) and only its remainder is read a second time.  Everything
 *    else takes slower element-wise multi-pass kernels.  Results are identical up to rounding order.
 */
#ifndef A3PO_H
#define A3PO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    A3PO_F32 = 0,
    A3PO_BF16 = 1,
    A3PO_DTYPE_INT_RANGE_ = 0x7fffffff /* not a dtype: makes every int a value of the type, so that an */
                                       /* unknown code reaches the library's own check (A3PO_E_DTYPE) */
} a3po_dtype;

enum {
    A3PO_OK = 0,
    A3PO_E_NULL = -1,        /* a required pointer is NULL                          */
    A3PO_E_SIZE = -2,        /* T < 0, V <= 0, ld < V, T or ld > 2^40, V >= 2^31,   */
                             /* G <= 0, S % G != 0, ...                             */
    A3PO_E_DTYPE = -3,       /* dtype is not A3PO_F32 / A3PO_BF16                   */
    A3PO_E_ALIGN = -4,       /* logits / dlogits / workspace base not aligned       */
    A3PO_E_WORKSPACE = -5,   /* workspace_bytes below a3po_workspace_bytes(...)     */
    A3PO_E_LAUNCH = -6,      /* the HIP runtime rejected a launch                   */
    A3PO_E_VALUE = -7        /* clip_eps not in [0,1), NaN scalar, ...              */
};

/* Run statistics of one loss call (the paper tracks importance-weight extrema and the
 * number of clipped tokens as stability evidence, Section 4.2.2).  Device resident.
 * iw_min / iw_max are +inf / -inf when no token enters the mean. */
typedef struct {
    int64_t n_tokens;             /* tokens that enter the mean: mask != 0 and id valid */
    int64_t n_clipped;            /* of those, tokens whose clipped branch is the min   */
    int64_t n_bad_index;          /* mask != 0 but chosen id outside [0,V)              */
    int64_t n_negative_staleness; /* counted tokens with current_version < version      */
    float iw_min, iw_max;         /* extrema of pi_prox/pi_behav over counted tokens    */
    float entropy_mean;           /* mean policy entropy over counted tokens when the   */
                                  /* call computed entropies, otherwise 0               */
    float reserved;               /* written as 0                                       */
} a3po_stats;

/* How the proximal log-prob of Eq. 2 is obtained (the three methods the paper compares,
 * Section 4.2: "loglinear", "recompute", "sync"). */
typedef enum {
    A3PO_PROX_INTERP = 0, /* A-3PO: Eq. 3 with the staleness coefficient of Eq. 4             */
    A3PO_PROX_GIVEN = 1,  /* decoupled loss with a proximal log-prob the caller computed      */
                          /* (an extra forward pass); versions are ignored                    */
    A3PO_PROX_BEHAV = 2   /* proximal = behaviour policy: the coupled objective of Eq. 1      */
                          /* (importance weight 1); versions are ignored                      */
} a3po_prox_mode;

/* Optional extras of a3po_loss_fwd_bwd_ex.  Host struct, read during the call only.
 * A zero-filled struct selects the behaviour of a3po_loss_fwd_bwd. */
typedef struct {
    int32_t prox_mode;         /* a3po_prox_mode                                                */
    int32_t accumulate;        /* 0: loss_out / stats_out are overwritten.  1: this call's share is     */
                               /* added to what they hold (micro-batches of one gradient update: sums   */
                               /* add, extrema and the entropy mean merge); they must have been written */
                               /* by an earlier call on the same stream                                 */
    const float *logp_prox_in; /* device [T]; required for A3PO_PROX_GIVEN, ignored otherwise   */
    float *entropy_out;        /* device [T], nullable: policy entropy -sum_j p_j log p_j of    */
                               /* each counted row (0 for rows that do not enter the loss),     */
                               /* accumulated in the same pass over the row as the log-sum-exp  */
    float *iw_out;             /* device [T], nullable: pi_prox/pi_behav per token (0 if not    */
                               /* counted)                                                      */
    uint8_t *clipped_out;      /* device [T], nullable: 1 where the clipped branch is the min   */
    void *event_before_rows;   /* hipEvent_t, nullable: recorded on `stream` immediately before */
    void *event_after_rows;    /* and after the vocabulary-wide row kernel (never waited on)    */
    const float *denom_dev;    /* device [1], nullable: when set, replaces the `denom` argument (read   */
                               /* on the stream, so a count produced by a3po_count_tokens needs no host */
                               /* round trip); a value <= 0 selects this call's own token count         */
} a3po_loss_options;

enum { A3PO_WS_LOSS_FWD_BWD = 0, A3PO_WS_FUSED_LMHEAD = 1, A3PO_WS_FUSED_LMHEAD_LOSS = 2 };

/* Bytes of device workspace the given entry point needs (256-byte aligned base). */
size_t a3po_workspace_bytes(int which, int64_t T, int64_t V, int64_t H);

/* Static description of an error code. */
const char *a3po_strerror(int code);

/*
 * log pi_theta(y_t | s_t) from logits: log-softmax over the vocabulary at temperature 1
 * (the paper samples at temperature 1.0, Section 4.1) and a gather of the chosen token.
 *   lse_t = log sum_j exp z[t,j],  logp_out[t] = z[t,y_t] - lse_t      (fp32 accumulate)
 * lse_out (nullable) [T] float.  chosen_logit_out (nullable) [T] elements of dtype `dt`:
 * the stored z[t,y_t] copied bit for bit.  A chosen id outside [0,V) gives logp 0 and a
 * zero chosen logit; lse is still written.  Reads T*V elements once.
 * Logits may be -inf (entries that cannot be sampled: probability exactly 0).  Accuracy of lse and
 * logp: 1e-5 (1 + |value|) whatever the magnitude of the logits (differences z - max are taken before
 * any scaling, and logp is (z_y - max) - log sum exp(z - max), not z_y - lse).
 */
int a3po_token_logprobs(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                        const int32_t *chosen, float *logp_out, float *lse_out,
                        void *chosen_logit_out, void *stream);

/*
 * a3po_token_logprobs plus the policy entropy of every row (the stability curve of Section
 * 4.2.2, Fig. 4), accumulated in the same single read of the row:
 *   entropy_out[t] = -sum_j p_j log p_j = lse_t - sum_j p_j z[t,j],   p_j = exp(z[t,j] - lse_t).
 * entropy_out [T] float, required; the other arguments as above.
 */
int a3po_token_logprobs_entropy(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                                const int32_t *chosen, float *logp_out, float *lse_out,
                                void *chosen_logit_out, float *entropy_out, void *stream);

/*
 * Staleness-aware proximal log-prob, Eq. 3 with the coefficient of Eq. 4 (argument order
 * of Listing 1: behaviour log-probs, current log-probs, per-token behaviour versions,
 * current version):
 *   d = current_version - versions[t];  alpha = 1/d if d >= 1 else 1;
 *   logp_prox_out[t] = alpha * logp_behav[t] + (1 - alpha) * logp_theta[t]     (fp32)
 * d is the exact integer difference (any int32 versions, so up to 2^32 - 1), converted to fp32 once:
 * alpha is the correctly rounded 1/d for d <= 2^24 and within one fp32 ulp of it beyond.
 * alpha_out (nullable) [T] float.  All arrays [T].
 */
int a3po_proximal_interp(const float *logp_behav, const float *logp_theta,
                         const int32_t *versions, int32_t current_version, int64_t T,
                         float *logp_prox_out, float *alpha_out, void *stream);

/*
 * Group-normalised advantages (GRPO; Section 4.1 "group reward normalization"): groups are
 * G consecutive sequences, A_s = (R_s - mean_g R) / (std_g R + eps_adv) with the population
 * standard deviation; adv_out[t] = A_{seq_id[t]}.  rewards [S] float, S % G == 0,
 * seq_id [T] int32 in [0,S) (an id outside gives advantage 0), adv_out [T] float.
 */
int a3po_grpo_advantages(const float *rewards, int64_t S, int32_t G, float eps_adv,
                         const int32_t *seq_id, int64_t T, float *adv_out, void *stream);

/*
 * The fused path: token log-probs, Eq. 4 / Eq. 3 proximal log-prob, the decoupled clipped
 * objective of Eq. 2 with a masked token mean, and the gradient of the loss with respect to
 * the logits, reading each live row once and writing each gradient row once.
 *
 *   lt = log pi_theta (as above), lp = alpha lb + (1-alpha) lt (held fixed: the proximal
 *   policy is a frozen anchor, Section 2.2), iw = exp(lp - lb), r = exp(lt - lp),
 *   obj = iw * min(r A, clip(r, 1-eps, 1+eps) A),   loss = -(1/N) sum_t m_t obj_t,
 *   N = denom if denom > 0 else the number of counted tokens; N == 0 => loss 0, dlogits 0.
 *   g_t = -(m_t/N) iw A r if the un-clipped branch is the min (ties included) else 0,
 *   dlogits[t,j] = g_t * ([j == y_t] - exp(z[t,j] - lse_t)).
 *
 * logits / dlogits: dtype `dt`, stride ld; dlogits may alias logits exactly (in place),
 * any other overlap is undefined.  Rows that are masked, have an invalid id, are clipped or
 * have A == 0 get an all-zero gradient row; masked / invalid rows are not read and get
 * logp_out = logp_prox_out = 0.  Padding columns V..ld-1 are neither read nor written.
 * chosen, versions [T] int32; logp_behav, advantages [T] float; loss_mask [T] uint8.
 * logp_out [T], logp_prox_out [T] (nullable), loss_out [1], stats_out (nullable): device.
 * workspace: a3po_workspace_bytes(A3PO_WS_LOSS_FWD_BWD, T, V, 0) bytes, 256-byte aligned,
 * private to the call until the stream has passed it.  The loss is reduced in a fixed order:
 * identical inputs give bit-identical outputs.
 */
int a3po_loss_fwd_bwd(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                      const int32_t *chosen, const float *logp_behav,
                      const int32_t *versions, int32_t current_version,
                      const float *advantages, const uint8_t *loss_mask,
                      float clip_eps, float denom,
                      void *dlogits, float *logp_out, float *logp_prox_out,
                      float *loss_out, a3po_stats *stats_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * a3po_loss_fwd_bwd for callers that cannot allocate or hand over device memory beyond inputs and outputs
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is an
 * array built into the library, A3PO_NOALLOC_MAX_TOKENS tokens' worth (about 6 MB of every GPU the library
 * runs on, held until the process ends).  The call allocates and frees nothing; its first use on a device looks
 * up that device's copy of the array (one hipGetSymbolAddress).  Arguments, results and error codes are those
 * of a3po_loss_fwd_bwd (same kernels: bit-identical outputs); T above A3PO_NOALLOC_MAX_TOKENS returns
 * A3PO_E_SIZE.  Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU race (issue
 * them on one stream, or order the streams).  Nothing the array holds is carried from one call to the next.
 */
#define A3PO_NOALLOC_MAX_TOKENS 131072
int a3po_loss_fwd_bwd_noalloc(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                              const int32_t *chosen, const float *logp_behav,
                              const int32_t *versions, int32_t current_version,
                              const float *advantages, const uint8_t *loss_mask,
                              float clip_eps, float denom,
                              void *dlogits, float *logp_out, float *logp_prox_out,
                              float *loss_out, a3po_stats *stats_out, void *stream);

/*
 * a3po_loss_fwd_bwd with the extras of a3po_loss_options (opt == NULL: no extras):
 *  - the two baselines the paper compares against through the same kernels: a caller-supplied
 *    proximal log-prob ("recompute"; lp = logp_prox_in[t], iw = exp(lp - lb), r = exp(lt - lp)) and
 *    the coupled objective of Eq. 1 ("sync"; lp = lb, so iw = 1 and r = exp(lt - lb));
 *    `versions` may be NULL for both;
 *  - per-token policy entropy (Section 4.2.2 tracks it) from the same read of the row, and its
 *    mean over counted tokens in stats_out->entropy_mean;
 *  - per-token importance weights and clip decisions, for histograms beyond the extrema and the
 *    count in a3po_stats;
 *  - two events around the row kernel, so a caller can time that kernel without a profiler.
 *  - mini-batch support: a denominator read from device memory and accumulation of loss and
 *    statistics over the micro-batches of one gradient update (see a3po_plan_microbatches).
 * Returns A3PO_E_VALUE for an unknown prox_mode or an accumulate flag other than 0 / 1, A3PO_E_NULL
 * when A3PO_PROX_GIVEN comes without logp_prox_in.
 */
int a3po_loss_fwd_bwd_ex(const void *logits, a3po_dtype dt, int64_t T, int64_t V, int64_t ld,
                         const int32_t *chosen, const float *logp_behav,
                         const int32_t *versions, int32_t current_version,
                         const float *advantages, const uint8_t *loss_mask,
                         float clip_eps, float denom,
                         void *dlogits, float *logp_out, float *logp_prox_out,
                         float *loss_out, a3po_stats *stats_out,
                         void *workspace, size_t workspace_bytes, void *stream,
                         const a3po_loss_options *opt);

/*
 * Histogram of a per-token quantity, for the distributions behind the stability statistics of
 * Section 4.2.2 (Fig. 5 plots only the extrema of the importance weight, Fig. 6 only the number of
 * clipped tokens): e.g. values = iw_out of a3po_loss_fwd_bwd_ex with select = loss_mask (all counted
 * tokens) or select = clipped_out (the clipped ones), or values = entropy_out.
 *   values [T] float, device.  select [T] uint8, device, nullable: token t is counted iff
 *   select[t] != 0 (NULL: every token).  edges [nbins + 1] float, DEVICE, non-decreasing
 *   (not checked; with unsorted edges every value still lands in some slot).
 *   counts_out [nbins + 3] int64, device: [0] values below edges[0]; [1 + k] values with
 *   edges[k] <= v < edges[k+1]; [nbins + 1] values >= edges[nbins]; [nbins + 2] NaNs.
 *   accumulate = 0 overwrites counts_out, 1 adds to it (micro-batches of one update).
 * Values are compared with the edges as stored, so the counts are exact integers.
 * 1 <= nbins <= A3PO_HIST_MAX_BINS, else A3PO_E_SIZE; accumulate not 0 / 1: A3PO_E_VALUE.
 * T == 0 is legal (counts_out is cleared unless accumulating).
 */
#define A3PO_HIST_MAX_BINS 1024
int a3po_histogram(const float *values, const uint8_t *select, int64_t T, const float *edges, int32_t nbins,
                   int32_t accumulate, int64_t *counts_out, void *stream);

/* ---- mini-batches (Section 4.1: a training step makes 4 gradient updates, one per mini-batch, and a
 * forward/backward pass holds at most 10,240 tokens) -------------------------------------------------
 *
 * Layout: sequences are packed back to back without padding, so row t of the logits is token t of the
 * packed stream and sequence s owns rows [offset_s, offset_s + seq_len[s]).  A mini-batch is a
 * contiguous run of sequences and one gradient update; it is cut into micro-batches, contiguous runs
 * of whole sequences whose token total stays within the budget.  Each micro-batch is one call of
 * a3po_loss_fwd_bwd_ex on its row range with the mini-batch's token count as denominator
 * (a3po_count_tokens -> a3po_loss_options.denom_dev) and accumulate = 1 after the first, so that loss,
 * statistics and gradients add up to exactly those of the mini-batch evaluated in one piece.
 */

/*
 * Plans the split.  HOST pointers.  seq_len [S] (>= 0).  Mini-batch k (0 <= k < n_minibatches) holds
 * sequences [k*S/n, (k+1)*S/n) (integer division; empty when S < n).  Inside a mini-batch, sequences are
 * taken in order and a new micro-batch starts whenever the next sequence would push the token total
 * over max_tokens; a sequence longer than max_tokens gets a micro-batch of its own.  Empty sequences
 * ride along with their neighbours.
 * Outputs: micro_first_seq [capacity + 1]: micro-batch i holds sequences micro_first_seq[i] ..
 * micro_first_seq[i+1]-1; micro_minibatch [capacity]: the mini-batch it belongs to; *n_micro_out: how
 * many micro-batches there are.  capacity >= S + n_minibatches always suffices.
 * Returns A3PO_E_SIZE for S < 0, n_minibatches <= 0, max_tokens <= 0, a negative length or a capacity
 * that is too small (nothing useful is written then).
 */
int a3po_plan_microbatches(const int64_t *seq_len, int64_t S, int32_t n_minibatches, int64_t max_tokens,
                           int64_t *micro_first_seq, int32_t *micro_minibatch, int64_t capacity,
                           int64_t *n_micro_out);

/*
 * Number of tokens that enter the loss (mask != 0 and 0 <= chosen < V) among T tokens, written as a
 * float to denom_out [1] (device; the denominator of a mini-batch) and, if count_out is not NULL, as
 * an integer to count_out [1] (device).  Exact up to 2^24 tokens as a float.
 */
int a3po_count_tokens(const int32_t *chosen, const uint8_t *loss_mask, int64_t T, int64_t V,
                      float *denom_out, int64_t *count_out, void *stream);

/* ---- vocabulary-sharded variant (a tensor-parallel LM head: each shard holds a column slice) ------
 *
 * The vocabulary [0,V) is split into P contiguous column ranges [v0_p, v0_p + Vs_p); shard p holds
 * logits_shard_p [T, Vs_p] (row stride ld_p; a column slice of a full matrix is such a shard with
 * base = full + v0_p and ld = the full stride).  Forward: every shard reduces its columns to one
 * partial per token (a3po_shard_partials); the P partial arrays are gathered into one [P, T] array
 * (the exchange between shards is the caller's) and merged (a3po_shard_combine) into the same lse /
 * log pi_theta / entropy the unsharded entry points give.  Backward: every shard writes its slice of
 * the gradient from the merged values (a3po_shard_loss_bwd), evaluating Eq. 2 - Eq. 4 per token
 * exactly as a3po_loss_fwd_bwd does, so loss and statistics come out identical on every shard.
 * chosen[t] is always the GLOBAL token id.
 */
typedef struct {
    float max;           /* max_j z[t, j] over the shard's columns                            */
    float sum_exp;       /* sum_j exp(z[t, j] - max)                                          */
    float chosen_logit;  /* z[t, chosen[t]] if the shard owns that column, else 0             */
    float sum_exp_z;     /* sum_j exp(z[t, j] - max) * z[t, j]   (for the entropy)            */
} a3po_shard_partial;

/* partial_out [T].  logits_shard: dtype dt, [T, Vs], stride ld >= Vs (16-byte aligned base and stride for the vector path); v0 >= 0 is
 * the global id of the shard's first column.  Reads T * Vs elements once. */
int a3po_shard_partials(const void *logits_shard, a3po_dtype dt, int64_t T, int64_t Vs, int64_t ld,
                        const int32_t *chosen, int64_t v0, a3po_shard_partial *partial_out, void *stream);

/* partials [P, T] (shard-major), merged in ascending shard order.  V = full vocabulary size (a chosen id
 * outside [0,V) gives logp 0).  logp_out [T]; lse_out, entropy_out [T] nullable. */
int a3po_shard_combine(const a3po_shard_partial *partials, int32_t P, int64_t T, const int32_t *chosen, int64_t V,
                       float *logp_out, float *lse_out, float *entropy_out, void *stream);

/* Loss and this shard's gradient slice from the merged log pi_theta and lse (both [T], as written by
 * a3po_shard_combine):  dlogits_shard[t, j] = g_t ([v0 + j == chosen[t]] - exp(z[t, j] - lse[t])).
 * Per-token arguments, loss_out, stats_out, workspace (A3PO_WS_LOSS_FWD_BWD size) and error codes as in
 * a3po_loss_fwd_bwd; dlogits_shard may alias logits_shard exactly.  Exactly the T x Vs elements of the
 * slice are written: when the slice is a column range of a wider matrix, its neighbours' columns and the
 * padding of the rows stay as they are.  opt (nullable): prox_mode,
 * logp_prox_in, iw_out and clipped_out are honoured; entropy_out and the events are ignored. */
int a3po_shard_loss_bwd(const void *logits_shard, a3po_dtype dt, int64_t T, int64_t Vs, int64_t ld, int64_t v0,
                        int64_t V, const int32_t *chosen, const float *logp_theta, const float *lse,
                        const float *logp_behav, const int32_t *versions, int32_t current_version,
                        const float *advantages, const uint8_t *loss_mask, float clip_eps, float denom,
                        void *dlogits_shard, float *logp_prox_out, float *loss_out, a3po_stats *stats_out,
                        void *workspace, size_t workspace_bytes, void *stream, const a3po_loss_options *opt);

/*
 * Token log-probs straight from hidden states and the LM-head weight (the 8B-shape fused
 * workload; the paper itself starts from log pi_theta and never mentions the projection):
 *   z[t, v] = sum_k hidden[t, k] * weight[v, k]   (bfloat16 inputs, fp32 accumulate on the matrix
 *   cores),  lse_t = log sum_v exp z[t, v],  logp_out[t] = z[t, chosen[t]] - lse_t.
 * The [T, V] logits are never written to memory: each 256 x 256 tile is folded into a running
 * (max, sum) per token as it leaves the matrix cores.
 * hidden [T, H] and weight [V, H]: row-major, contiguous, bfloat16, 16-byte aligned; H must be a
 * positive multiple of 64, at most 2^20 (A3PO_E_SIZE otherwise).  chosen [T] int32; an id outside [0,V) gives logp 0 (lse still written).
 * logp_out [T] float, lse_out [T] float (nullable).
 * workspace: a3po_workspace_bytes(A3PO_WS_FUSED_LMHEAD, T, V, H) bytes, 256-byte aligned.
 * The first call in a process raises the kernel's dynamic LDS limit (one hipFuncSetAttribute, done once, safe
 * against concurrent first calls from several host threads).
 */
int a3po_fused_lmhead_logprob(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                              const int32_t *chosen, float *logp_out, float *lse_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole path from hidden states: LM-head projection, then everything a3po_loss_fwd_bwd does,
 * then the gradient contracted back through the projection:
 *   z = hidden weight^T,  loss / log-probs / statistics as in a3po_loss_fwd_bwd (same arguments),
 *   dhidden[t, :] = sum_v dlogits[t, v] weight[v, :],   dweight[v, :] = sum_t dlogits[t, v] hidden[t, :].
 * Only tokens that enter the loss (mask != 0, valid id) are projected: every other token has log-prob 0 and a
 * zero row of dhidden by definition and costs nothing beyond that row's zero fill.  The counted tokens are
 * compacted on the device and taken in chunks of 8,192.  The log-sum-exp and the log-probs of a chunk are
 * folded from fp32 tiles as they leave the matrix cores, exactly as in a3po_fused_lmhead_logprob (both entry
 * points give the same log pi_theta up to rounding order); the same tiles are also kept in fp32 inside the
 * workspace, for that chunk only, and the gradient rows dlogits are formed from them in fp32 and rounded once
 * to bfloat16, the operand type of the matrix cores.  The three contractions are this library's own kernel
 * (bfloat16 operands, fp32 accumulation); dweight is contracted over up to 65,536 counted tokens at a time and
 * rounded to bfloat16 once: straight from the accumulators when T <= 65,536, else after summing the contractions
 * in fp32.
 * hidden, dhidden [T, H]; weight, dweight [V, H]: row-major, contiguous, bfloat16, 16-byte
 * aligned; H a positive multiple of 64, at most 2^20; V a multiple of 8 below 2^21; T below 2^22
 * (A3PO_E_SIZE otherwise).  Per-token arguments and outputs as in a3po_loss_fwd_bwd.
 * workspace: a3po_workspace_bytes(A3PO_WS_FUSED_LMHEAD_LOSS, T, V, H) bytes, 256-byte aligned: W^T, the gathered
 * hidden rows and their transpose, a chunk of logits (fp32) and of its gradient, the vocabulary-major gradient of
 * up to 65,536 tokens, and beyond that many tokens an fp32 accumulator of dweight - about 2 V H + 6 T H +
 * 6 * 8192 V + 2 V min(T, 65536) (+ 4 V H) bytes, 30 GB at T = 65,536, H = 4,096, V = 151,936.
 */
int a3po_fused_lmhead_loss_fwd_bwd(const void *hidden, const void *weight, int64_t T, int64_t H, int64_t V,
                                   const int32_t *chosen, const float *logp_behav,
                                   const int32_t *versions, int32_t current_version,
                                   const float *advantages, const uint8_t *loss_mask,
                                   float clip_eps, float denom,
                                   void *dhidden, void *dweight, float *logp_out, float *logp_prox_out,
                                   float *loss_out, a3po_stats *stats_out,
                                   void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* A3PO_H */
