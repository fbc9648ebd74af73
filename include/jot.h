/*
 * jot.h -- C ABI of the JoT token-finalization pass for AMD Instinct MI355X (gfx950).
 *
 * One call to jot_step() performs, for one denoising step n of a masked-diffusion decoder,
 * what the paper's Algorithm 1 does between the computation of the logits and the transfer schedule:
 *
 *   for every examined (still masked, eligible) position i:
 *     pi = softmax(l^i) over the vocabulary, no temperature          (Section 4.1, Confidence Metric)
 *     p1, p2 = two largest probabilities, a = argmax                   (Section 4.1)
 *     conf  = p1 / (p2 + eps)                                          (Eq. 2)   [or p1, or p1 - p2]
 *     w     = sum of gamma^|i-j| over resolved j, 1 <= |i-j| <= D      (Eq. 3)
 *     phi   = min(1, w / w_max), w_max = 2 * sum_{d=1..D} gamma^d      (Eq. 4)
 *     tau_i = tau_max - (tau_max - tau_min) * phi                      (Eq. 5)
 *     conf >= tau_i  =>  token[i] = a, position leaves the masked set  (Eq. 6)
 *   all decisions of a step use the mask as it was when the step began (Algorithm 1: M_n is
 *   formed once per step); finalization is uncapped; prompt tokens count as resolved context
 *   and, with semi-autoregressive decoding, only the current block is examined
 *   (Section 4.2, Implementation details).
 *
 * Only the logit rows of examined positions are read.  Frozen positions cost no memory traffic.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the caller.  The library never
 *     allocates or frees device memory; its working memory is the caller's workspace.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.  jot_init_state()
 *     and jot_step() only enqueue work on that stream and return; they do not synchronise
 *     (jot_init_state synchronises once).  A state must always be used with the same stream,
 *     or the caller must order the streams itself.
 *   - Return value 0 = success, negative = one of JOT_ERR_*.  Arguments are validated on the
 *     host before any device work, so a failing call has no effect on the device.
 *   - A state belongs to the HIP device that was current in jot_init_state(); later calls on it
 *     must be made with the same device current (else JOT_ERR_WRONG_DEVICE).
 *   - Calls on the same state must not overlap (one thread at a time); different states are
 *     independent.
 *   - Indices: a canvas position is the flattened index b*L + i, 0 <= b < B, 0 <= i < L.
 *     Steps are numbered from 1.
 */
#ifndef JOT_H
#define JOT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jot_state jot_state;      /* opaque, host memory, created by jot_init_state, freed by jot_release */

typedef enum { JOT_F32 = 0, JOT_BF16 = 1 } jot_dtype;

/* Confidence signal compared with tau_i.  All three come from the same (p1, p2). */
typedef enum {
    JOT_CONF_RATIO   = 0,   /* Eq. 2: p1 / (p2 + eps); thresholds on the ratio scale (e.g. 90, 30)   */
    JOT_CONF_MAXPROB = 1,   /* p1; thresholds in [0, 1]                                                */
    JOT_CONF_PROBGAP = 2    /* p1 - p2; thresholds in [0, 1]                                           */
} jot_conf_mode;

enum {
    JOT_OK                      =  0,
    JOT_ERR_INVALID_ARG         = -1,
    JOT_ERR_NULL_POINTER        = -2,
    JOT_ERR_UNSUPPORTED_DTYPE   = -3,
    JOT_ERR_WORKSPACE_TOO_SMALL = -4,
    JOT_ERR_MISALIGNED          = -5,
    JOT_ERR_HIP                 = -6,
    JOT_ERR_NO_DEVICE           = -7,
    JOT_ERR_NO_MEMORY           = -8,   /* host allocation failed */
    JOT_ERR_WRONG_DEVICE        = -9,   /* the current HIP device is not the one the state was created on */
    JOT_ERR_TOO_LARGE           = -10   /* jot_step_static: the problem does not fit the library's fixed scratch array */
};

typedef struct {
    int32_t B, L, V;          /* batch rows, canvas length INCLUDING the prompt, vocabulary size (>= 2) */
    int32_t dtype;            /* jot_dtype of the logits                                                */
    int32_t conf_mode;        /* jot_conf_mode                                                          */
    float   tau_max, tau_min; /* Eq. 5; tau_min <= tau_max                                              */
    float   gamma;            /* Eq. 3 decay, in (0, 1]                                                 */
    int32_t D;                /* Eq. 3 window radius, 0..32; 0 switches spatial modulation off (phi=0)  */
    float   eps;              /* Eq. 2; the paper uses 1e-12; >= 0                                      */
    int32_t gen_start;        /* first generation position (= prompt length), 0..L; blocks count from it*/
    int32_t block_size;       /* 0: every masked position is examined each step (fully parallel decode);
                                 >0: only the masked positions of each row's current block, i.e. the
                                 block [gen_start + k*block_size, gen_start + (k+1)*block_size) that
                                 holds the row's lowest masked position                                 */
} jot_params;

/* Bytes of device workspace a state with these parameters needs (multiple of 256).
 * <0: JOT_ERR_* (invalid parameters).  Host only. */
int64_t jot_workspace_bytes(const jot_params* p);

/*
 * Create a state.  Copies the initial canvas into the workspace and builds the first list of
 * examined positions.  Synchronises `stream` once before returning.
 *   out            : receives the state (host object; free with jot_release)
 *   workspace_dev  : device memory, 256-byte aligned, >= jot_workspace_bytes(p) bytes; must stay
 *                    valid and untouched by the caller for the life of the state
 *   tokens_dev     : [B, L] int32, row-major; tokens of resolved positions (value at a masked
 *                    position is ignored and later overwritten by the finalized token)
 *   masked_dev     : [B, L] uint8, 1 = masked ([M]), 0 = resolved (prompt or already decoded)
 */
int jot_init_state(jot_state** out, const jot_params* p,
                   void* workspace_dev, int64_t workspace_bytes,
                   const int32_t* tokens_dev, const uint8_t* masked_dev, void* stream);

/*
 * One finalization pass (step n = number of jot_step calls so far on this state, from 1).
 *   logits_dev : logits of the whole canvas, element (b, i, v) at
 *                logits_dev[b*stride_b + i*stride_l + v]; strides in ELEMENTS; V contiguous.
 *                Must be 16-byte aligned, and stride_b, stride_l must keep every row 16-byte
 *                aligned.  Read-only; only rows of examined positions are touched, so rows of
 *                frozen positions need not hold valid data.
 *   -inf logits are allowed (probability 0), and so are very negative finite fill values
 *   (-1e9, -1e30, -FLT_MAX): they contribute 0.  A row holding NaN or +inf, or only -inf, or
 *   whose largest logit lies outside [-4e6, 4e6], has no softmax here: the position is left
 *   masked and counted by jot_anomaly_count().
 * Asynchronous: returns after enqueueing on `stream`.  With no examined position left it is a
 * no-op on the canvas (Algorithm 1 would have left the loop).
 */
int jot_step(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l, void* stream);

/*
 * jot_step plus the decoder's transfer schedule (Section 3.2 "Iterative Sampling"; Section 4.2
 * "Interaction with transfer schedules", "Implementation details": the schedule reveals the k
 * most confident masked positions, confidence = max_v pi_v, and the early-exit mask is OR-ed on
 * top of it, uncapped).  Per batch row b, of the positions examined this step the
 *     k_b = min(#rows with a softmax, n_transfer[b] + floor(transfer_frac * #examined in row b))
 * with the largest p1 (equal p1: lower position first) are finalized with their argmax token, in
 * addition to every position that passes Eq. 6.  In block mode the schedule, like the early
 * exit, acts inside the row's current block.
 *   n_transfer_dev : [B] int32 DEVICE array (a per-step entry of a precomputed schedule), or NULL
 *                    for all zeros; negative totals count as 0
 *   transfer_frac  : in [0, 1]; e.g. 1 - s/t for decoders that reveal num_masked * (1 - s/t),
 *                    1.0 on the last step reveals everything that has a softmax
 * jot_step(...) is jot_step_scheduled(..., NULL, 0.0f, ...).  Same asynchrony and errors.
 */
int jot_step_scheduled(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                       const int32_t* n_transfer_dev, float transfer_frac, void* stream);

/*
 * jot_step_scheduled with sampling-based finalization (Section 4.1, "Early-Exit Decision": the
 * finalized token may be sampled from the predicted distribution instead of taking the argmax).
 * Which positions are finalized is decided exactly as in jot_step_scheduled; a finalized position
 * (b, i) gets the token drawn from pi by inverse-CDF sampling at the uniform number
 * uniforms_dev[b*L + i]: the first vocabulary index whose cumulative probability exceeds it.
 *   uniforms_dev : [B, L] float DEVICE array of numbers in [0, 1), drawn by the caller for this
 *                  step; read only at finalized positions.  NULL = argmax finalization.
 * Rows finalized in this step are read a second time (once per position over a whole decode).
 * If the cumulative sum never exceeds the uniform number (a number within rounding of 1, or one
 * that is not below 1), the token is the last one with a non-zero probability: the cumulative
 * probability reaches 1 there.
 */
int jot_step_sampled(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                     const int32_t* n_transfer_dev, float transfer_frac, const float* uniforms_dev,
                     void* stream);

/*
 * The general step.  `opt` gathers the optional rules of a step; NULL or an all-zero struct is
 * plain jot_step.  jot_step, jot_step_scheduled and jot_step_sampled are shorthands for it.
 *
 * Row-wide early commit (enable_global_gap != 0): the global rule the paper's related-work section
 * describes for Prophet -- once the top-2 confidence gap clears a threshold, every remaining
 * masked position is finalized at once.  Here, per batch row: if the MEAN of the top-2 logit gaps
 * l_(1) - l_(2) over the row's examined positions that have a softmax is >= global_gap, all of
 * those positions are finalized this step (argmax, or sampled if uniforms_dev is given), OR-ed
 * with the early exit and the schedule.  A staged threshold (e.g. 7.5 / 5 / 2.5 as decoding
 * progresses) is simply a different global_gap per call.
 *
 * KL stability rule (enable_kl != 0): the per-token rule the related-work section describes for
 * KLASS -- the KL divergence between the distributions of consecutive steps marks predictions
 * that have stopped moving (Section 6.1 quotes its two thresholds).  An examined position is
 * stable if the previous step examined it too (and it had a softmax there),
 * D(pi_now || pi_prev) <= kl_threshold, and p1 >= kl_min_prob; stable positions are finalized,
 * OR-ed with the other rules.  The step then streams two logit tensors:
 *   prev_logits_dev : the tensor that was `logits_dev` of the PREVIOUS step of this state, kept
 *                     alive and unchanged by the caller (ping-pong two buffers); same element
 *                     type, strides and alignment as logits_dev.  Its log-normalizers were stored
 *                     by that step; passing anything else gives meaningless divergences.
 * On the first step, and for positions the previous step did not examine (a block that has just
 * become current), there is no previous distribution and the rule does not fire.  Vocabulary
 * entries whose probability underflows binary32 relative to the row maximum (below ~1e-38) count
 * as probability 0 in the divergence.
 *
 * Compact logits (logits_compact != 0): for decoders that apply the output projection to the
 * examined positions only.  logits_dev then holds one row per entry of jot_active_list(), in
 * that order: row r at logits_dev[r*stride_l + v], r < jot_active_count(); stride_b is ignored.
 * Same alignment rules.  Cannot be combined with enable_kl (the previous step's rows are in the
 * previous step's order): JOT_ERR_INVALID_ARG.
 */
typedef struct {
    const int32_t* n_transfer_dev;   /* transfer schedule, see jot_step_scheduled; may be NULL      */
    float          transfer_frac;    /* in [0, 1]                                                   */
    const float*   uniforms_dev;     /* sampling, see jot_step_sampled; NULL = argmax               */
    int32_t        enable_global_gap;/* != 0: apply the row-wide early-commit rule this step        */
    float          global_gap;       /* its threshold (finite)                                      */
    int32_t        enable_kl;        /* != 0: apply the KL stability rule this step                 */
    const void*    prev_logits_dev;  /* the previous step's logits (required if enable_kl)          */
    float          kl_threshold;     /* tau_KL >= 0                                                 */
    float          kl_min_prob;      /* tau_conf in [0, 1]                                          */
    int32_t        logits_compact;   /* != 0: logits_dev is [jot_active_count(), V], see above      */
} jot_step_options;

int jot_step_ex(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                const jot_step_options* opt, void* stream);

/*
 * One finalization pass that allocates nothing, for callers that cannot allocate: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  It is jot_step
 * without a state object: the canvas comes in and goes out through the caller's arrays, and the
 * working memory (partial results, counters, lists, the bit image of the mask) is a fixed array
 * inside the library, JOT_STATIC_MAX_WORKSPACE bytes on every GPU the library runs on, held until
 * the process ends.  No device or host memory is allocated or freed, no event is created, nothing
 * is synchronised: the call only enqueues kernels on `stream`.
 *   p              : as for jot_init_state; jot_workspace_bytes(p) must not exceed
 *                    JOT_STATIC_MAX_WORKSPACE, else JOT_ERR_TOO_LARGE (about 26 000 canvas positions
 *                    B*L; the vocabulary size does not matter)
 *   logits_dev, stride_b, stride_l : as for jot_step
 *   tokens_dev     : [B, L] int32, in and out: finalized positions receive their token
 *   masked_dev     : [B, L] uint8, in and out: finalized positions are cleared
 *   active_out_dev : [B*L] int32, out: the positions a next step would examine, ascending b*L+i
 *   n_active_out_dev : int64, out: how many of them
 * The step is numbered 1 (no state is carried from call to call).  Every call on a GPU uses that
 * GPU's one array: calls that overlap on one GPU (different streams or threads) race, the caller
 * must order them.  The first call on a device looks up the array's address and the launch shapes;
 * make it outside stream capture.
 */
#define JOT_STATIC_MAX_WORKSPACE (4 << 20)
int jot_step_static(const jot_params* p, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                    int32_t* tokens_dev, uint8_t* masked_dev, int32_t* active_out_dev,
                    int64_t* n_active_out_dev, void* stream);

/* Algorithm 1's loop test: the size of the masked set M_n the NEXT step would examine (0 = decoding
 * finished; in block mode, the masked positions of the current blocks).  Waits for the work enqueued
 * so far on this state.  <0: JOT_ERR_*. */
int64_t jot_active_count(jot_state* s);

/* The same number without waiting: the count stored by the last step that has COMPLETED on the
 * device, and in *steps_done (may be NULL) how many steps have completed.  A decode loop can enqueue
 * the next forward pass, poll this until *steps_done reaches the number of steps it has enqueued, and
 * so overlap the test with other work.  Never blocks on the device. */
int64_t jot_active_count_poll(const jot_state* s, int32_t* steps_done);

/* After steps that were enqueued under stream capture (and are replayed as a HIP graph on a stream
 * the library never saw), the waiting calls above wait for the whole device.  Tell the library which
 * stream the replays run on: it records an event there (not under capture) and the waiting calls
 * wait for that event instead.  Call it after each replay whose results are to be read. */
int jot_wait_on_stream(jot_state* s, void* stream);

/* Number of steps completed on this state (n of Algorithm 1's loop), counted on the device, so it is
 * right for steps replayed from a captured graph as well.  Waits like jot_active_count. */
int32_t jot_step_index(jot_state* s);

/* Rows skipped so far because they had no softmax.  Waits like jot_active_count. */
int64_t jot_anomaly_count(jot_state* s);

/*
 * Device views into the workspace.  Pointers stay valid until the workspace is freed; the
 * contents are those of the last enqueued step once its stream work has completed.
 */
const int32_t* jot_tokens(const jot_state* s);        /* [B, L] the canvas x of Algorithm 1           */
const uint8_t* jot_masked(const jot_state* s);        /* [B, L] 1 = still [M] (membership in M_n)     */
const int32_t* jot_commit_step(const jot_state* s);   /* [B, L] step n at which Eq. 6 (or an optional
                                                         rule) finalized the position, 0 = not (yet)  */
/* Algorithm 1's masked set M_n for the next step, as a list: [jot_active_count] ascending b*L+i
 * (in block mode restricted to the current blocks, Section 4.2).  Waits like jot_active_count (the
 * list is double buffered; which half is current is device state). */
const int32_t* jot_active_list(jot_state* s);
/* Every finalization (Eq. 6: x^i <- argmax, i leaves M; or a token chosen by an optional rule) in
 * order: triples (step, b*L+i, token), steps non-decreasing, positions ascending within a step.
 * *n receives the number of triples (waits like jot_active_count). */
const int32_t* jot_commit_log(jot_state* s, int64_t* n);

/*
 * Per-position results of the LAST step, aligned with the list that step examined
 * (jot_examined_list, length *n = number of examined positions; waits like jot_active_count):
 * token = argmax_v pi_v and p1, p2 = the two largest probabilities (Section 4.1, Confidence Metric),
 * conf = the confidence of Eq. 2 (or the selected other signal), tau = tau_i of Eq. 5 (from w of
 * Eq. 3 and phi of Eq. 4).  For rows without a softmax conf is NaN.
 */
const int32_t* jot_examined_list(jot_state* s, int64_t* n);
const int32_t* jot_last_token(const jot_state* s);
const int32_t* jot_last_final_token(const jot_state* s);  /* token written if finalized: argmax or sample */
const float*   jot_last_conf(const jot_state* s);
const float*   jot_last_p1(const jot_state* s);
const float*   jot_last_p2(const jot_state* s);
const float*   jot_last_tau(const jot_state* s);
/* per examined position: bit 0 = passed Eq. 6, bit 1 = picked by the transfer schedule,
 * bit 2 = finalized by the row-wide early-commit rule, bit 3 = stable under the KL rule */
const uint8_t* jot_last_flags(const jot_state* s);
/* per examined position: the top-2 LOGIT gap l_(1) - l_(2) that the row-wide rule averages
 * (+inf if only one logit is finite) */
const float*   jot_last_gap(const jot_state* s);
/* per examined position: D(pi_now || pi_prev) of a step run with enable_kl; NaN where the position
 * has no previous distribution or no softmax, and after steps run without the rule */
const float*   jot_last_kl(const jot_state* s);

/*
 * Optional timing of the vocabulary-reduction kernel (the one that reads the logits):
 * when enabled, jot_step brackets that kernel with HIP events on `stream`; the events of the
 * last JOT_PROFILE_RING steps are kept.  jot_profile_read waits for step `step` (1-based, one of
 * the last JOT_PROFILE_RING steps enqueued while profiling was on) and returns that kernel's
 * duration in milliseconds in *vocab_reduce_ms.
 */
#define JOT_PROFILE_RING 64
int jot_profile_enable(jot_state* s, int on);
int jot_profile_read(jot_state* s, int32_t step, float* vocab_reduce_ms);

/* Free the host object and its pinned host counters (device memory is the caller's).  Waits for
 * the steps enqueued on this state to finish first; NULL is a no-op. */
void jot_release(jot_state* s);

const char* jot_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* JOT_H */
