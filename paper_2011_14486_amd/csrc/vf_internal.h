// Internal declarations of libvf (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "vf.h"

// candidates per partial-argmin slot (one slot per scoring workgroup)
#define VF_PART 128
// (value, id) pairs in the static scratch array of vf_score_static: one per scoring workgroup
#define VF_STATIC_PARTS 65536
// size of one packed decision context (see vf_sched_dev.h)
#define VF_DECPACK_DWORDS 428

// Where the scorers put their per-workgroup (value, id) minima when the context's own
// growable buffers must not be used (nullable everywhere it is taken): `cap` pairs.
struct vf_partbuf {
  float *val;
  int32_t *idx;
  size_t cap;
};

struct vf_packed_model {
  // fp32 path: the caller's blob copied as is
  float *w_f32 = nullptr;
  float *w_f32t = nullptr;  // fp32 MLPs: every layer's matrix transposed, [k][N rounded up to 16] (zeros in the padding)
  size_t n_floats = 0;
  // bf16 path: matrices repacked into MFMA A-fragment order, biases and the last
  // layer's vector as fp32
  uint16_t *w_pack = nullptr;      // all packed matrices back to back
  size_t pack_off[8] = {0};        // element offset of each matrix in w_pack
  float *aux = nullptr;            // biases / head vector, fp32
  size_t aux_off[8] = {0};         // element offset of each layer's bias in aux
  // bf16 MLPs whose hidden layers all have 512 (fast_rt = 2) or 1024 (fast_rt = 4)
  // units: the same matrices once more, ordered as one contiguous fragment stream
  // per wave over all hidden layers
  uint16_t *w_stream = nullptr;
  size_t wave_stride = 0;          // 16-byte units between the streams of two waves
  int fast_rt = 0;
  // 64 or 256 input rows (the search's feature layouts): only rows 16..55 and 59 depend on
  // the candidate.  The stream with the first layer cut to k-steps 1..3 (rows 16..63)
  uint16_t *w_stream_fold = nullptr;
  size_t wave_stride_fold = 0;
  // recurrent network wired to the search: [W_ih | W_hh] transposed, bf16 values as fp32, [64+H][4H]
  float *w_seqT = nullptr;
};

struct vf_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  int last_hip = 0;

  bool has_space = false, has_pipeline = false, has_model = false;
  vf_space space;
  int64_t M = 0, Mpad = 0;
  int S = 0, B = 0;
  int n_sched = 0;

  // device tables, all int32 unless noted
  int32_t *d_space = nullptr;   // [65]
  int32_t *d_stages = nullptr;  // [B][S][16]
  int32_t *d_intr = nullptr;    // [B][S][16] intrinsic block of every stage
  int32_t *d_suffix = nullptr;  // [B][S][2]  sums of macs / points over later stages
  int32_t *d_states = nullptr;  // [B][S][16]
  int32_t *d_cf = nullptr;      // [B][S][64] committed core features
  int32_t *d_prefix = nullptr;  // [B][S+1][2] sums of total_macs / bytes_written over committed stages
  int32_t *d_cids = nullptr;    // [B][S]
  float *d_vals = nullptr;      // [B][S]
  int32_t *d_alive = nullptr;   // [B] 0 once a stage of the problem found no winner
  int32_t *d_err = nullptr;     // [1] set by a forced commit of an invalid candidate
  unsigned long long *d_stat = nullptr;  // [2] ids scored by the fused step / valid ones, while profiling
  int32_t *d_forced = nullptr;  // [B][S] staging for vf_set_state
  uint32_t *d_decpack = nullptr; // [B][VF_DECPACK_DWORDS] decision context of stage dec_stage
  int dec_stage = -1;            // stage d_decpack was built for, -1: none
  uint32_t *d_decpack2 = nullptr; // second context buffer (behind the first in the same allocation), for chained layers
  // chained layers of a greedy schedule (vfk_greedy_chain): every fused launch but the first also
  // takes the decision of the stage before it
  bool chain_on = false;
  int chain_prev = -1;           // stage whose decision the next launch takes, -1: none
  int chain_par = 0;             // which context buffer / partial-minima set the next launch writes

  // beam search: a second set of state tables (the survivors of a layer are written
  // there, then the two sets swap), masked scores, selection scratch
  int32_t *d_alt_states = nullptr, *d_alt_cf = nullptr, *d_alt_prefix = nullptr, *d_alt_cids = nullptr;
  float *d_alt_vals = nullptr;
  int32_t *d_alt_alive = nullptr;
  float *d_scores = nullptr; size_t score_elems = 0;   // [B][Mpad]
  float *d_tk_val = nullptr; int32_t *d_tk_idx = nullptr; size_t tk_elems = 0;  // chunk partials
  float *d_sel_val = nullptr; int32_t *d_sel_idx = nullptr;  // [B] survivors (value, beam*Mpad+cid)
  int32_t *d_sel_n = nullptr;    // [2]: survivors of this layer, live schedules so far
  // recurrent value network wired to the search: per-problem tables and prefix state
  // of the recurrence (two sets: beam search writes the survivors' state into the other)
  float *d_seq_G = nullptr;                       // [B][S][4H] gate inputs of unscheduled stages
  float *d_seq_h[2] = {nullptr, nullptr};         // [B][H] h of the last committed stage (bf16 values)
  float *d_seq_c[2] = {nullptr, nullptr};         // [B][H] its cell state
  float *d_seq_P[2] = {nullptr, nullptr};         // [B][4H] biases + W_hh h: gates of the next step
  float *d_seq_hs[2] = {nullptr, nullptr};        // [B] head predictions summed over the committed stages
  int32_t *d_seq_list = nullptr, *d_seq_count = nullptr;  // [B][Mpad] valid ids of the decision, [B] their number
  int seq_stage = -1;                             // committed stages folded into the state, -1: none valid
  int seq_cur = 0;                                // which set is current
  // exploration noise added to the scores in the argmin scan of step / greedy calls
  float noise_eps = 0.0f;
  uint64_t noise_seed = 0;
  int32_t noise_first = 0;
  std::vector<vf_stage> h_stages;  // host copy of the stage records
  bool beam_checked = false;       // all slots verified to hold the same pipeline

  vf_model model;
  vf_packed_model pm;

  // scratch, grown on demand
  int32_t *d_feat = nullptr; size_t feat_elems = 0;
  float *d_act[2] = {nullptr, nullptr}; size_t act_elems = 0;
  float *d_pval = nullptr; int32_t *d_pidx = nullptr; size_t part_elems = 0;
  unsigned int *d_team = nullptr; size_t team_elems = 0;  // team meetings: counters, error flag, per-member minima
  int32_t *h_team_err = nullptr;  // pinned: the error flag of the last team launch, copied back after it
  // the last whole-schedule launch, until somebody has looked at its error flag: the event behind
  // the flag's copy, the layers the call was asked for, the state epoch it ran in
  hipEvent_t ev_whole = nullptr;
  bool whole_pending = false;
  int whole_first = 0, whole_last = -1;
  uint64_t state_epoch = 0, whole_epoch = 0;  // state_epoch: bumped whenever the schedule state is replaced
  // the last occupancy answer for the whole-schedule kernel (kernel, dynamic LDS -> workgroups per CU)
  mutable const void *occ_kern = nullptr;
  mutable size_t occ_smem = 0;
  mutable int occ_blocks = 0;
  unsigned int wait_rounds = 1u << 22;  // bound of the waits between workgroups that share a problem
  int32_t *d_wlist = nullptr; size_t wlist_elems = 0;  // [B][Mpad] id lists of the whole-schedule launch

  vf_partbuf static_parts = {nullptr, nullptr, 0};  // this device's static scratch array (vf_score_static)

  hipEvent_t ev0 = nullptr, ev1 = nullptr;

  // per-kernel timing (benchmarks): event pairs recorded around launches
  bool profiling = false;
  std::vector<hipEvent_t> prof_pairs[3];  // begin, end, begin, end, ...
  std::vector<hipEvent_t> prof_free;
};

// Brackets one kernel launch with events when profiling is on.
struct vf_prof_scope {
  vf_ctx *c;
  int which;
  hipEvent_t e1 = nullptr;
  vf_prof_scope(vf_ctx *ctx, int w) : c(ctx), which(w) {
    if (!c->profiling) return;
    hipEvent_t e0 = take();
    e1 = take();
    if (!e0 || !e1) { e1 = nullptr; return; }
    (void)hipEventRecord(e0, c->stream);
    c->prof_pairs[which].push_back(e0);
    c->prof_pairs[which].push_back(e1);
  }
  ~vf_prof_scope() {
    if (e1) (void)hipEventRecord(e1, c->stream);
  }
  hipEvent_t take() {
    if (!c->prof_free.empty()) {
      hipEvent_t e = c->prof_free.back();
      c->prof_free.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

#define VF_HIP(ctx, call)                          \
  do {                                             \
    hipError_t e_ = (call);                        \
    if (e_ != hipSuccess) {                        \
      (ctx)->last_hip = (int)e_;                   \
      return VF_EHIP;                              \
    }                                              \
  } while (0)

// ---- vf_sched.hip: enumeration, featurization, commit ----
// A packed bf16 MLP with uniform hidden width, as the fused scoring kernels take it.
struct vf_fast_dev {
  int L;
  int dims[8];
  const uint4 *w_stream;   // per wave: [layer][k step][row tile r][lane] fragments
  size_t wave_stride;      // in uint4
  const float *aux;
  int naux;                // floats in aux (biases of all layers, output vector)
  size_t bias_off[8];
  size_t wl_off;
  int k0;                  // k-steps of the first layer present in w_stream ...
  int k0ofs;               // ... starting with this one (fold: steps 1..3 = input rows 16..63)
  const uint4 *w_full;     // nullable (fold): the stream with the whole first layer, for the rows that the
  size_t wave_stride_full; // candidates of a decision share (k-steps 0, 3 and, with 256 inputs, 4..15)
};
void vfk_fast_dev(const vf_ctx *c, bool generating, vf_fast_dev *fd, int *ks, int *NC);

int vfk_setup_tables(vf_ctx *c);
int vfk_reset_state(vf_ctx *c);
// stages first.. become unscheduled again (tables as after committing stages 0..first-1)
int vfk_rewind(vf_ctx *c, int first);
int vfk_enumerate(vf_ctx *c, int stage, uint32_t *dec, uint8_t *valid, int32_t *n_valid);
int vfk_featurize(vf_ctx *c, int stage, int32_t *feat);
// reduce the per-workgroup partial minima of every problem, report and optionally commit
int vfk_commit_from_partials(vf_ctx *c, int stage, int nparts, int commit, int32_t *best_cid,
                             float *best_val);
int vfk_commit_forced(vf_ctx *c, int stage);
// builds d_decpack for `stage` unless it is already there
int vfk_prepare(vf_ctx *c, int stage);

// ---- vf_score.hip: value networks and argmin ----
int vfk_pack_model(vf_ctx *c, const float *weights_dev);
void vfk_free_model(vf_ctx *c);
// Scores nprob problems of M candidates each: x + p*prob_stride is [F][ld].
// use_valid_row: row 16 of x is the validity flag (invalid -> +inf).
// noise_stage >= 0: the context's exploration noise for that layer is added before the scan.
// Writes scores (nullable, [nprob][ld_scores]) and the partial minima
// (ctx->d_pval / d_pidx, [nprob][nparts], ids local to the problem).
int vfk_score_mlp(vf_ctx *c, const int32_t *x, int64_t prob_stride, int nprob, int64_t M, int64_t ld,
                  int use_valid_row, float *scores, int64_t ld_scores, int *nparts_out, int noise_stage,
                  const vf_partbuf *parts = nullptr);
// Enumerate + featurize + score + partial argmin of one stage in a single kernel (bf16
// MLPs of uniform hidden width whose input width is the space's F).
bool vfk_can_fuse_step(const vf_ctx *c);
int vfk_whole_team(const vf_ctx *c);
bool vfk_seq_model(const vf_ctx *c);
void vfk_seq_free(vf_ctx *c);
int vfk_seq_sync(vf_ctx *c, int stage);
int vfk_seq_advance(vf_ctx *c, int stage);
int vfk_seq_advance_beam(vf_ctx *c, int stage);
int vfk_seq_step(vf_ctx *c, int stage, float *scores, int64_t ld_scores, int noise_stage, int *nparts_out);
int vfk_greedy_whole(vf_ctx *c, int first, int last);
int vfk_step_fused(vf_ctx *c, int stage, int *nparts_out);
// Algorithm 1 over stages first..last with one launch per layer (the fused scorer also decides
// the stage before it) and one commit at the end; VF_ESTATE if the model or space does not
// take the fused path.
bool vfk_can_chain(const vf_ctx *c);
int vfk_greedy_chain(vf_ctx *c, int first, int last);
// k_commit on given partial minima and a given context buffer (nullable: rebuilt from the tables)
int vfk_commit_from(vf_ctx *c, int stage, int nparts, const float *pval, const int32_t *pidx, const uint32_t *decpack_cur);
// Scores of every candidate of `stage` for all problems into d_scores [B][Mpad]; invalid
// candidates and padding columns get +inf.
int vfk_step_scores(vf_ctx *c, int stage);
// beam search pieces (vf_sched.hip)
int vfk_beam_init(vf_ctx *c, int first_stage);
int vfk_beam_select_commit(vf_ctx *c, int stage);
int vfk_score_lstm(vf_ctx *c, const uint16_t *x, int64_t M, int T, float *scores, int *nparts_out,
                   const vf_partbuf *parts = nullptr);
int vfk_argmin_groups(vf_ctx *c, int64_t M, int nparts, int parts_per_group, int ngroups,
                      int32_t *best_idx, float *best_val, const vf_partbuf *parts = nullptr);
// The static scratch array of vf_score_static on the current device (looked up once per
// device), as a partial-minima buffer; VF_EHIP if the symbol's address cannot be had.
int vfk_static_parts(vf_ctx *c, vf_partbuf *out);
int vfk_ensure_parts(vf_ctx *c, size_t n);
