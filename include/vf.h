/*
 * libvf -- value-function-guided greedy scheduling on one AMD MI355X (gfx950).
 *
 * The library runs the hot loop of Algorithm 1 ("Scheduling") of "Value Function
 * Based Performance Optimization of Deep Learning Workloads" (arXiv 2011.14486):
 * for each layer L_i in scheduling order, enumerate the candidate states
 * C_i = CandidateActions(L_i, s_{i-1}), featurize each one, score it with the value
 * network V(s), keep the first minimum, commit it and go on.
 *
 * Every entry point takes plain pointers and sizes.  "host" pointers are ordinary
 * process memory and are copied before the call returns.  "dev" pointers are device
 * memory on the context's GPU, owned by the caller; the library enqueues work on the
 * HIP stream given to vf_create and returns without synchronising, so outputs are
 * valid once that stream has completed.  Calls on one context must not overlap.
 *
 * B independent scheduling problems ("batch") with the same number of stages S, the
 * same search space and the same value network can be held by one context; every
 * per-decision call then works on all B problems at once and every output has a
 * leading dimension B.  B = 1 is the single-network case of Algorithm 1.
 *
 * Return value: VF_OK (0) or a negative error code; no entry point throws or aborts.
 * "No candidate wins" (no valid candidate, or every score is NaN / +inf) is not an
 * error: Algorithm 1 then leaves s_i unset (v_i stays at infinity); it is reported
 * in-band as candidate id -1 with value +inf, and that problem's schedule ends there.
 */
#ifndef VF_H
#define VF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VF_OK = 0,
  VF_EINVAL = -1, /* bad argument, shape or descriptor                          */
  VF_ESTATE = -2, /* call out of order (stage not next, nothing set, bad prefix) */
  VF_ENOMEM = -3, /* host or device allocation failed                            */
  VF_EHIP = -4    /* a HIP call failed; vf_last_hip_error() has its status       */
};

/* stage kinds and compute_at levels */
enum { VF_CONV = 0, VF_DWCONV = 1, VF_POINTWISE = 2, VF_ADD = 3 };
enum { VF_ROOT = 0, VF_L1 = 1, VF_L2 = 2, VF_INLINE = 3 };
/* value-network kinds, arithmetic, vf_score input kinds */
enum { VF_MLP = 0, VF_LSTM = 1 };
enum { VF_FP32 = 0, VF_BF16 = 1 };
enum { VF_X_RAW_I32 = 0, VF_X_SEQ_BF16 = 1 };

typedef struct vf_ctx vf_ctx; /* opaque; owns the state tables and scratch buffers */

/* One layer of the network (Sec. 2: "NN with n layers L_1 ... L_n"), batch 1:
 * w[0] kind; w[1..3] output extents W, H, C; w[4] RC reduced input channels (C_in of
 * a CONV, else 1); w[5] KH; w[6] KW; w[7] stride; w[8] anchor = index of an
 * earlier-listed stage that consumes this stage's output (-1: none); w[9] number of
 * consumers; w[10], w[11] stages producing its inputs (-1: pipeline input);
 * w[12] bytes per element; w[13..15] zero.  Stages are listed in scheduling order. */
typedef struct { int32_t w[16]; } vf_stage;

/* A committed decision s_i and the loop structure it imposes (Sec. 2):
 * w[0..2] inner extents fx, fy, fc; w[3] loop-order index; w[4] vectorize; w[5]
 * parallel; w[6] compute_at level; w[7] store_at hoist; w[8..10] region extents per
 * instance Ex, Ey, Ec; w[11] instances; w[12..14] outer extents Ox, Oy, Oc;
 * w[15] 1 if the stage is scheduled, 0 otherwise (then the record is all zero). */
typedef struct { int32_t w[16]; } vf_state;

/* The candidate space: one digit per primitive of Table 1 (split x/y/c, reorder,
 * vectorize, parallel, compute_at, store_at) plus the machine-model constants used
 * by the features.  Candidate id, least significant digit first:
 * cid = ix + nf[0]*(iy + nf[1]*(ic + nf[2]*(iperm + nperm*(vec + nvec*(par +
 *       npar*(icat + ncat*isat)))))).                                           */
typedef struct {
  int32_t nf[3];      /* number of split factors for x, y, c (1..8)                */
  int32_t fac[3][8];  /* the factors (inner extents), each >= 1                    */
  int32_t nperm;      /* number of loop orders (1..8)                              */
  int32_t perm[8][3]; /* loop orders, outermost first, each a permutation of 0,1,2 */
  int32_t nvec, npar; /* 1 (off only) or 2 (off, on)                               */
  int32_t ncat;       /* number of compute_at levels offered (1..4)                */
  int32_t cat[4];     /* the levels, values VF_ROOT..VF_INLINE                     */
  int32_t nsat;       /* store_at hoist amounts 0..nsat-1 (1..3)                   */
  int32_t vlen, ncores, l1_bytes, l2_bytes; /* machine-model constants             */
  int32_t F;          /* features per candidate: 64 or 256                         */
} vf_space;

/* The value network V(s).  MLP: dims = F, h_1, ..., 1 with n_layers = number of
 * weight matrices (<= 7), ReLU between layers.  LSTM (Sec. 3.2): dims = F, H, 1 and
 * n_layers = 2: one LSTM layer whose per-timestep linear predictions are summed.
 * dtype VF_BF16: weights, inputs and hidden activations in bfloat16, sums in fp32. */
typedef struct {
  int32_t kind, n_layers, dims[8], dtype;
} vf_model;

/* ---- context ------------------------------------------------------------- */

/* Creates a context on GPU `device`; hip_stream is a hipStream_t (NULL = the default
 * stream).  The stream stays the caller's.  *out is NULL on failure. */
int vf_create(vf_ctx **out, int device, void *hip_stream);
/* Waits for the stream, frees everything the context owns.  NULL is allowed. */
void vf_destroy(vf_ctx *ctx);

/* Search space (host, copied).  Resets the scheduling state. */
int vf_set_space(vf_ctx *ctx, const vf_space *space_host);
/* stages_host[batch][n_stages] (host, copied): `batch` pipelines of n_stages layers
 * each.  Needs a space.  Resets the scheduling state to s_0 (nothing scheduled). */
int vf_set_pipeline(vf_ctx *ctx, const vf_stage *stages_host, int n_stages, int batch);
/* weights_dev: n_floats fp32 values in device memory, read during this call's stream
 * work and not kept: MLP  W_1[h_1][F], b_1[h_1], ..., W_L[1][h_{L-1}], b_L[1];
 * LSTM  W_ih[4H][F], W_hh[4H][H], b_ih[4H], b_hh[4H], w_head[H], b_head[1] with the
 * four gate blocks in the order i, f, g, o.  With VF_BF16 the library rounds the
 * matrices (and w_head) to bfloat16, ties to even; biases stay fp32.
 * VF_BF16 needs every MLP width except the last to be a multiple of 32 and at most
 * 1024 (LSTM: F and H multiples of 32, at most 256).  VF_LSTM supports VF_BF16 only.
 * Anything else is VF_EINVAL.
 * Which V the search calls (vf_argmin_step, vf_greedy_schedule, vf_beam_search) accept:
 * an MLP with dims[0] == space.F, applied to the feature column of a candidate state;
 * or an LSTM with dims[0] == 64, applied to the state as a sequence (Sec. 3.2): one
 * timestep per stage of the pipeline in scheduling order, a stage that is scheduled in
 * the state (committed before, or the candidate itself) gives its 64 core features, a
 * stage that is not gives its intrinsic block (rows 0..15) and zeros, all normalised;
 * V = the head applied to every timestep's hidden state, summed.  Any other model is
 * VF_EINVAL there (it can still be used with vf_score). */
int vf_set_model(vf_ctx *ctx, const vf_model *model_host, const float *weights_dev, size_t n_floats);

/* s_0 = InitialState of Algorithm 1: nothing scheduled. */
int vf_reset_state(vf_ctx *ctx);
/* Commits candidate cids_host[b][j] for stages j < n_scheduled of every problem b
 * (host, [batch][n_scheduled]) as if the greedy loop had chosen them.  Synchronises
 * the stream; VF_ESTATE if one of them is not a valid candidate (the state is then
 * reset to s_0). */
int vf_set_state(vf_ctx *ctx, const int32_t *cids_host, int n_scheduled);
/* Number of stages committed so far. */
int vf_n_scheduled(const vf_ctx *ctx);

/* M = product of the radices of the space; M_pad = M rounded up to 256.  0 if no
 * space is set. */
int64_t vf_dense_count(const vf_ctx *ctx);
int64_t vf_padded_count(const vf_ctx *ctx);

/* ---- the five steps of Algorithm 1 ---------------------------------------- */

/* C_i = CandidateActions(L_i, s_{i-1}) for stage i = `stage` <= vf_n_scheduled():
 * the dense id range [0, M) with a validity flag (Sec. 2: the options valid given
 * the loop structure of the scheduled layers).
 * dec_dev[batch][M_pad]: the eight digits of each id, 4 bits each, ix lowest.
 * valid_dev[batch][M_pad]: 1 / 0.  n_valid_dev[batch]: number of valid ids.
 * Entries M..M_pad-1 are written as zero.  Any output may be NULL. */
int vf_enumerate(vf_ctx *ctx, int stage, uint32_t *dec_dev, uint8_t *valid_dev, int32_t *n_valid_dev);

/* Features of every candidate state of stage `stage` (Sec. 3.2: intrinsic and
 * acquired features), raw non-negative integers saturating at 2^31-1, feature-major:
 * feat_dev[batch][F][M_pad].  Rows 0..15 intrinsic, 16..55 acquired (row 16 is the
 * validity flag), 56..63 context; with F = 256 rows 64..207 hold features 0..47 of
 * the three stages committed just before and rows 208..255 the intrinsic block of
 * the next three stages.  Invalid candidates keep rows 0..15 and 64..255 and have
 * zeros in rows 16..63; columns M..M_pad-1 are zero. */
int vf_featurize(vf_ctx *ctx, int stage, int32_t *feat_dev);

/* V(s) for M candidates, and optionally the scan "if V(s) < v_i" of Algorithm 1.
 * x_kind VF_X_RAW_I32 (MLP): x_dev is int32 [F][ld] raw features, candidate n in
 *   column n; they are normalised (piecewise-linear log2) inside.  ld >= M.
 * x_kind VF_X_SEQ_BF16 (LSTM): x_dev is bfloat16 [M][T][F] normalised per-stage
 *   feature sequences, ld = T.
 * scores_dev[M] (nullable) receives the values.  If best_idx_dev / best_val_dev are
 * not NULL they receive, for each consecutive block of `group` candidates (group = 0:
 * one block of all M; otherwise M is split into ceil(M/group) blocks and group must
 * be a multiple of 128), the smallest id with the minimal score and that score; a
 * candidate wins only if its score is strictly smaller, so NaN never wins; a block
 * with no winner gets -1 and +inf. */
int vf_score(vf_ctx *ctx, const void *x_dev, int32_t x_kind, int64_t M, int64_t ld, int32_t group,
             float *scores_dev, int32_t *best_idx_dev, float *best_val_dev);

/* vf_score for callers that cannot allocate device memory while they run: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results as vf_score, but the per-workgroup minima that
 * the scoring kernel leaves for the group scan live in a static device array of the
 * library (512 KiB per GPU, held until the process ends) instead of a buffer that grows on
 * demand: the call allocates and frees nothing (no per-kernel timing events either: the
 * call is not bracketed by vf_profile_enable).  Limits: VF_BF16 models only (VF_EINVAL for
 * VF_FP32, whose layer-by-layer kernels keep whole activation matrices in scratch), and at
 * most vf_score_static_max() candidates per call - 65536 workgroup tiles of 64 candidates
 * (LSTM, MLP wider than 512) or 128 (other MLPs) - else VF_EINVAL and nothing is launched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (other
 * streams, other contexts, other threads) race; calls in stream order on one stream do not. */
int vf_score_static(vf_ctx *ctx, const void *x_dev, int32_t x_kind, int64_t M, int64_t ld, int32_t group,
                    float *scores_dev, int32_t *best_idx_dev, float *best_val_dev);
/* Largest M vf_score_static accepts with the context's model (0: no model, or not VF_BF16). */
int64_t vf_score_static_max(const vf_ctx *ctx);

/* One iteration of the outer loop of Algorithm 1 for stage `stage` ==
 * vf_n_scheduled(): enumerate, featurize, score, argmin over the valid candidates.
 * best_cid_dev[batch], best_val_dev[batch] (nullable) receive the winners.  If
 * `commit` is non-zero the winners become s_i and the context advances. */
int vf_argmin_step(vf_ctx *ctx, int stage, int commit, int32_t *best_cid_dev, float *best_val_dev);

/* Algorithm 1 for stages first_stage..last_stage (first_stage == vf_n_scheduled()),
 * without host synchronisation between layers.  Outputs (all nullable):
 * out_states_dev[batch][S] the committed states s_1..s_n so far (all stages),
 * out_cids_dev[batch][S] the chosen candidate ids, out_values_dev[batch][S] their
 * values; entries of stages not scheduled yet are zero states, -1 and +inf.
 * With 24 or more problems (and a model whose tile fits the LDS) the layers run inside one
 * launch: with fewer problems than half the compute units several workgroups share a problem
 * from the start, with more a workgroup that has finished its own problems helps with the
 * ones still running; workgroups that share a problem meet once per layer with a bounded
 * wait.  Should such a wait ever run out (the GPU shared with work that never ends), the
 * launch still ends, and the problems it did not finish read -1 / +inf / zero state from the
 * first unfinished layer on.  The library learns of it when the stream has got there:
 * vf_sync_status waits for that and reports it; otherwise the next call that builds on the
 * context's schedule state (vf_greedy_schedule / vf_beam_search from first_stage > 0,
 * vf_argmin_step / vf_enumerate / vf_featurize for a stage > 0) waits for the verdict before
 * it does anything, and a call that starts from s_0 looks whether the verdict is in.
 * Whoever finds out returns VF_ESTATE after repairing what can be repaired: if the context
 * still holds that call's state, the layers it was asked for are run again with the launches
 * per layer, so that the tables are complete afterwards and
 * vf_greedy_schedule(first_stage = vf_n_scheduled()) fetches them. */
int vf_greedy_schedule(vf_ctx *ctx, int first_stage, int last_stage, vf_state *out_states_dev,
                       int32_t *out_cids_dev, float *out_values_dev);

/* Exploration noise (Sec. 3.1, BestSchedule(n, V_eps) of Algorithm 2: a small random
 * noise is added to the predictions so that repeated greedy runs cover different
 * schedules).  From now on vf_argmin_step and vf_greedy_schedule scan
 * V(s) + eps * u(seed, first_rollout + b, layer, candidate id) for problem b, with u in
 * [-1, 1) = (top 24 bits of the first Philox4x32-10 word of counter (id, layer,
 * rollout, 0) under key seed) * 2^-23 - 1, one fp32 multiply and one fp32 add; the
 * reported values are the noisy ones.  A batch of B copies of one network is thus B
 * different rollouts.  eps = 0 (the initial state) switches the noise off.  vf_score
 * and vf_beam_search never add noise.  VF_EINVAL for a negative or non-finite eps. */
int vf_set_noise(vf_ctx *ctx, float eps, uint64_t seed, int32_t first_rollout);

/* Beam search guided by V (Secs. 3.1 and 4.1 search with a beam as well, next to the
 * greedy scan; Algorithm 2 completes prefixes with it).  The context's `batch` problems
 * are the beam slots of ONE network: every slot must hold the same pipeline (else
 * VF_EINVAL) and the beam width is `batch` (at most 1024; batch * padded id count must stay
 * below 2^31).  Starts from problem 0's current schedule
 * (first_stage == vf_n_scheduled(); after vf_reset_state that is s_0); the other slots'
 * schedules are discarded.  Per layer every surviving partial schedule is extended by
 * every valid candidate, all extensions are scored, and the `batch` smallest scores
 * survive, ordered by (score, parent slot, candidate id); +inf and NaN never survive.
 * If a layer has no survivor the schedules found so far are kept and end there.
 * Outputs as vf_greedy_schedule, row j = j-th best schedule; unused rows are zero
 * states, -1, +inf.  n_beams_dev[1] (nullable) = number of schedules found.  Width 1
 * takes the same decisions as vf_greedy_schedule. */
int vf_beam_search(vf_ctx *ctx, int first_stage, int last_stage, vf_state *out_states_dev,
                   int32_t *out_cids_dev, float *out_values_dev, int32_t *n_beams_dev);

/* ---- diagnostics ---------------------------------------------------------- */

/* Static description of an error code. */
const char *vf_strerror(int code);
/* Status (hipError_t as int) of the last failed HIP call on this context, 0 if none. */
int vf_last_hip_error(const vf_ctx *ctx);
/* Time in milliseconds between two points recorded on the context's stream with HIP
 * events: vf_timer_start / vf_timer_stop enqueue the events, vf_timer_elapsed_ms
 * synchronises on the second one.  For benchmarks. */
int vf_timer_start(vf_ctx *ctx);
int vf_timer_stop(vf_ctx *ctx);
int vf_timer_elapsed_ms(vf_ctx *ctx, float *ms_host);
/* Per-kernel timing for benchmarks.  While enabled, vf_featurize, vf_score,
 * vf_argmin_step and vf_greedy_schedule bracket each launch of their featurize
 * (which = 0), scoring (1) and commit (2) kernels with HIP events on the context's
 * stream.  vf_profile_read synchronises, returns the summed duration and the number
 * of launches of one kind since the last read of that kind, and clears them. */
enum { VF_PROF_FEATURIZE = 0, VF_PROF_SCORE = 1, VF_PROF_COMMIT = 2 };
int vf_profile_enable(vf_ctx *ctx, int enable);
int vf_profile_read(vf_ctx *ctx, int which, double *total_ms_host, int64_t *launches_host);
/* While profiling is enabled the fused step of vf_argmin_step / vf_greedy_schedule /
 * vf_beam_search counts, over all problems of the batch, the candidate ids it pushed
 * through V and how many of them were valid candidates (Algorithm 1 evaluates V on the
 * candidates only; runs of ids that the compute_at / store_at digits alone rule out are
 * decided without the network and are not counted).  vf_profile_counts synchronises,
 * returns both counts since the last call and clears them.  Either pointer may be NULL. */
int vf_profile_counts(vf_ctx *ctx, int64_t *scored_host, int64_t *valid_host);
/* Waits until everything enqueued on the context's stream has run and reports how the last
 * whole-schedule launch of vf_greedy_schedule ended: VF_OK, or VF_ESTATE if one of its
 * bounded waits between workgroups ran out - then, if the context still holds that call's
 * state, the affected layers have been run again with the launches per layer before this
 * call returns, and the tables are complete (see vf_greedy_schedule). */
int vf_sync_status(vf_ctx *ctx);
/* Bound of the waits between the workgroups that share a problem inside a whole-schedule
 * launch of vf_greedy_schedule, in polling rounds (default 2^22, seconds); a helper's wait
 * for work starts over whenever a problem finishes anywhere, so a launch that is merely long
 * does not run it out.  A wait that reaches the bound gives up: the launch still ends, see
 * vf_greedy_schedule for what follows.  A bound of 0 makes every wait that cannot be
 * satisfied at once give up; meant for tests of that path. */
int vf_set_wait_limit(vf_ctx *ctx, unsigned int rounds);

#ifdef __cplusplus
}
#endif
#endif /* VF_H */
