// C ABI of libvf: argument checking, context tables, and the per-layer loop of
// Algorithm 1 as a sequence of kernel launches on the caller's stream.
#include <string.h>

#include <new>
#include <vector>

#include "vf_internal.h"

namespace {

bool space_ok(const vf_space *s) {
  for (int d = 0; d < 3; ++d) {
    if (s->nf[d] < 1 || s->nf[d] > 8) return false;
    for (int k = 0; k < s->nf[d]; ++k)
      if (s->fac[d][k] < 1) return false;
  }
  if (s->nperm < 1 || s->nperm > 8) return false;
  for (int p = 0; p < s->nperm; ++p) {
    int seen = 0;
    for (int k = 0; k < 3; ++k) {
      if (s->perm[p][k] < 0 || s->perm[p][k] > 2) return false;
      seen |= 1 << s->perm[p][k];
    }
    if (seen != 7) return false;
  }
  if (s->nvec < 1 || s->nvec > 2 || s->npar < 1 || s->npar > 2) return false;
  if (s->ncat < 1 || s->ncat > 4) return false;
  for (int k = 0; k < s->ncat; ++k)
    if (s->cat[k] < VF_ROOT || s->cat[k] > VF_INLINE) return false;
  if (s->nsat < 1 || s->nsat > 3) return false;
  if (s->vlen < 1 || s->ncores < 1 || s->l1_bytes < 0 || s->l2_bytes < 0) return false;
  if (s->F != 64 && s->F != 256) return false;
  return true;
}

int64_t dense_count(const vf_space *s) {
  int64_t m = 1;
  const int32_t r[8] = {s->nf[0], s->nf[1], s->nf[2], s->nperm, s->nvec, s->npar, s->ncat, s->nsat};
  for (int k = 0; k < 8; ++k) m *= r[k];
  return m;
}

bool stages_ok(const vf_stage *st, int S, int B) {
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < S; ++j) {
      const int32_t *w = st[(size_t)b * S + j].w;
      if (w[0] < VF_CONV || w[0] > VF_ADD) return false;
      for (int k = 1; k <= 7; ++k)
        if (w[k] < 1) return false;
      if (w[8] < -1 || w[8] >= j) return false;
      if (w[9] < 0 || w[12] < 1) return false;
    }
  return true;
}

bool model_ok(const vf_model *m, size_t n_floats) {
  if (m->dtype != VF_FP32 && m->dtype != VF_BF16) return false;
  if (m->kind == VF_MLP) {
    if (m->n_layers < 1 || m->n_layers > 7) return false;
    size_t n = 0;
    for (int l = 0; l <= m->n_layers; ++l)
      if (m->dims[l] < 1) return false;
    if (m->dims[m->n_layers] != 1) return false;
    for (int l = 0; l < m->n_layers; ++l) n += (size_t)m->dims[l] * m->dims[l + 1] + m->dims[l + 1];
    if (n != n_floats) return false;
    if (m->dtype == VF_BF16)
      for (int l = 0; l < m->n_layers; ++l)
        if (m->dims[l] % 32 != 0 || m->dims[l] > 1024) return false;
    return true;
  }
  if (m->kind == VF_LSTM) {
    if (m->dtype != VF_BF16 || m->n_layers != 2 || m->dims[2] != 1) return false;
    const int F = m->dims[0], H = m->dims[1];
    if (F < 32 || F % 32 != 0 || F > 256 || H < 32 || H % 32 != 0 || H > 256) return false;
    size_t n = (size_t)4 * H * F + (size_t)4 * H * H + (size_t)8 * H + H + 1;
    return n == n_floats;
  }
  return false;
}

void free_pipeline(vf_ctx *c) {
  vfk_seq_free(c);
  void *ps[] = {c->d_stages, c->d_intr, c->d_suffix, c->d_states, c->d_cf, c->d_prefix,
                c->d_cids,   c->d_vals, c->d_alive,  c->d_forced, c->d_decpack};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  c->d_stages = c->d_intr = c->d_suffix = c->d_states = c->d_cf = c->d_prefix = c->d_cids = nullptr;
  c->d_alive = c->d_forced = nullptr;
  c->d_vals = nullptr;
  c->d_decpack = nullptr;
  c->d_decpack2 = nullptr;
  c->dec_stage = -1;
  void *alt[] = {c->d_alt_states, c->d_alt_cf, c->d_alt_prefix, c->d_alt_cids, c->d_alt_vals, c->d_alt_alive,
                 c->d_sel_val,    c->d_sel_idx, c->d_sel_n};
  for (void *p : alt)
    if (p) (void)hipFree(p);
  c->d_alt_states = c->d_alt_cf = c->d_alt_prefix = c->d_alt_cids = c->d_alt_alive = nullptr;
  c->d_alt_vals = nullptr;
  c->d_sel_val = nullptr;
  c->d_sel_idx = c->d_sel_n = nullptr;
  c->has_pipeline = false;
  c->S = c->B = c->n_sched = 0;
}

template <typename T>
int dev_alloc(vf_ctx *c, T *&p, size_t n) {
  void *q = nullptr;
  hipError_t e = hipMalloc(&q, (n ? n : 1) * sizeof(T));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    c->last_hip = (int)e;
    return e == hipErrorOutOfMemory ? VF_ENOMEM : VF_EHIP;
  }
  p = (T *)q;
  return VF_OK;
}

int ensure_feat(vf_ctx *c) {
  size_t want = (size_t)c->B * c->space.F * c->Mpad;
  if (want <= c->feat_elems) return VF_OK;
  if (c->d_feat) {
    VF_HIP(c, hipStreamSynchronize(c->stream));
    VF_HIP(c, hipFree(c->d_feat));
    c->d_feat = nullptr;
    c->feat_elems = 0;
  }
  int rc = dev_alloc(c, c->d_feat, want);
  if (rc == VF_OK) c->feat_elems = want;
  return rc;
}

// enumerate + featurize + score + argmin (+ commit) for one stage, all problems
// V is defined on the states of this context's pipeline: an MLP over the feature rows of
// the search space, or the recurrent network over 64 values per stage
bool model_fits(const vf_ctx *c) {
  return (c->model.kind == VF_MLP && c->model.dims[0] == c->space.F) || vfk_seq_model(c);
}

int step(vf_ctx *c, int stage, int commit, int32_t *best_cid, float *best_val) {
  if (vfk_seq_model(c)) {
    int nparts = 0;
    int rc = vfk_seq_step(c, stage, nullptr, 0, stage, &nparts);
    if (rc != VF_OK) return rc;
    rc = vfk_commit_from_partials(c, stage, nparts, commit, best_cid, best_val);
    if (rc == VF_OK && commit) rc = vfk_seq_advance(c, stage);
    return rc;
  }
  if (vfk_can_fuse_step(c)) {
    // features are produced and consumed inside one kernel and never reach HBM
    int nparts = 0;
    int rc = vfk_step_fused(c, stage, &nparts);
    if (rc != VF_OK) return rc;
    return vfk_commit_from_partials(c, stage, nparts, commit, best_cid, best_val);
  }
  int rc = ensure_feat(c);
  if (rc != VF_OK) return rc;
  rc = vfk_featurize(c, stage, c->d_feat);
  if (rc != VF_OK) return rc;
  int nparts = 0;
  rc = vfk_score_mlp(c, c->d_feat, (int64_t)c->space.F * c->Mpad, c->B, c->M, c->Mpad, 1, nullptr, 0, &nparts, stage);
  if (rc != VF_OK) return rc;
  return vfk_commit_from_partials(c, stage, nparts, commit, best_cid, best_val);
}

int settle_whole(vf_ctx *c, bool wait);

struct DeviceGuard {
  int prev = -1;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != dev) (void)hipSetDevice(dev);
    else prev = -1;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

// Looks at the outcome of the last whole-schedule launch, once.  wait = false: only if the
// launch has finished (otherwise later).  A launch in which a bounded wait between workgroups
// ran out has left some problems' schedules incomplete (unscheduled layers read -1 / +inf /
// zero state): if the context still holds that call's state, its layers are run again here,
// with the launches per layer, so that the tables end up complete; VF_ESTATE either way, so
// that the caller learns of it.
int settle_whole(vf_ctx *c, bool wait) {
  if (!c->whole_pending) return VF_OK;
  if (wait) {
    VF_HIP(c, hipEventSynchronize(c->ev_whole));
  } else {
    const hipError_t q = hipEventQuery(c->ev_whole);
    if (q == hipErrorNotReady) { (void)hipGetLastError(); return VF_OK; }
    VF_HIP(c, q);
  }
  c->whole_pending = false;
  if (!c->h_team_err || *c->h_team_err == 0) return VF_OK;
  *c->h_team_err = 0;
  if (c->state_epoch == c->whole_epoch && c->n_sched == c->whole_last + 1) {
    int rc = vfk_rewind(c, c->whole_first);
    if (rc != VF_OK) return rc;
    c->n_sched = c->whole_first;
    for (int i = c->whole_first; i <= c->whole_last; ++i) {
      rc = step(c, i, 1, nullptr, nullptr);
      if (rc != VF_OK) return rc;
      c->n_sched = i + 1;
    }
  }
  return VF_ESTATE;
}

}  // namespace

extern "C" {

int vf_create(vf_ctx **out, int device, void *hip_stream) {
  if (!out) return VF_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return VF_EINVAL;
  vf_ctx *c = new (std::nothrow) vf_ctx();
  if (!c) return VF_ENOMEM;
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  DeviceGuard g(device);
  int rc = dev_alloc(c, c->d_space, sizeof(vf_space) / 4);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_err, 1);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_stat, 2);
  if (rc == VF_OK && hipMemsetAsync(c->d_stat, 0, 16, c->stream) != hipSuccess) rc = VF_EHIP;
  if (rc == VF_OK) rc = vfk_static_parts(c, &c->static_parts);  // address of this device's static scratch
  if (rc == VF_OK && hipEventCreate(&c->ev0) != hipSuccess) rc = VF_EHIP;
  if (rc == VF_OK && hipEventCreate(&c->ev1) != hipSuccess) rc = VF_EHIP;
  if (rc != VF_OK) {
    vf_destroy(c);
    return rc;
  }
  *out = c;
  return VF_OK;
}

void vf_destroy(vf_ctx *c) {
  if (!c) return;
  DeviceGuard g(c->device);
  (void)hipStreamSynchronize(c->stream);
  free_pipeline(c);
  vfk_free_model(c);
  void *ps[] = {c->d_space, c->d_err,  c->d_stat, c->d_wlist, c->d_team, c->d_feat,   c->d_act[0], c->d_act[1],
                c->d_pval,  c->d_pidx, c->d_scores, c->d_tk_val, c->d_tk_idx};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  if (c->h_team_err) (void)hipHostFree(c->h_team_err);
  if (c->ev0) (void)hipEventDestroy(c->ev0);
  if (c->ev1) (void)hipEventDestroy(c->ev1);
  if (c->ev_whole) (void)hipEventDestroy(c->ev_whole);
  for (auto &v : c->prof_pairs)
    for (hipEvent_t e : v) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->prof_free) (void)hipEventDestroy(e);
  delete c;
}

int vf_set_space(vf_ctx *c, const vf_space *s) {
  if (!c || !s || !space_ok(s)) return VF_EINVAL;
  int64_t M = dense_count(s);
  if (M < 1 || M > (1 << 30)) return VF_EINVAL;
  DeviceGuard g(c->device);
  // the pipeline tables depend on nothing in the space, but the state does
  VF_HIP(c, hipStreamSynchronize(c->stream));
  c->space = *s;
  c->M = M;
  c->Mpad = (M + 255) / 256 * 256;
  VF_HIP(c, hipMemcpyAsync(c->d_space, &c->space, sizeof(vf_space), hipMemcpyHostToDevice, c->stream));
  VF_HIP(c, hipStreamSynchronize(c->stream));
  c->has_space = true;
  if (c->has_pipeline) return vf_reset_state(c);
  return VF_OK;
}

int vf_set_pipeline(vf_ctx *c, const vf_stage *st, int S, int B) {
  if (!c || !st || S < 1 || B < 1 || S > 4096 || (int64_t)S * B > (1 << 24)) return VF_EINVAL;
  if (!c->has_space) return VF_ESTATE;
  if (!stages_ok(st, S, B)) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipStreamSynchronize(c->stream));
  free_pipeline(c);
  c->S = S;
  c->B = B;
  const size_t n = (size_t)S * B;
  int rc = dev_alloc(c, c->d_stages, n * 16);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_intr, n * 16);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_suffix, n * 2);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_states, n * 16);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_cf, n * 64);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_prefix, (size_t)B * (S + 1) * 2);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_cids, n);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_vals, n);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_alive, (size_t)B);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_forced, n);
  if (rc == VF_OK) rc = dev_alloc(c, c->d_decpack, (size_t)2 * B * VF_DECPACK_DWORDS);
  if (rc == VF_OK) c->d_decpack2 = c->d_decpack + (size_t)B * VF_DECPACK_DWORDS;
  if (rc != VF_OK) {
    free_pipeline(c);
    return rc;
  }
  c->h_stages.assign(st, st + n);
  c->beam_checked = false;
  VF_HIP(c, hipMemcpyAsync(c->d_stages, st, n * sizeof(vf_stage), hipMemcpyHostToDevice, c->stream));
  VF_HIP(c, hipStreamSynchronize(c->stream));  // the host array may go away after return
  rc = vfk_setup_tables(c);
  if (rc != VF_OK) return rc;
  c->has_pipeline = true;
  return vf_reset_state(c);
}

int vf_set_model(vf_ctx *c, const vf_model *m, const float *weights_dev, size_t n_floats) {
  if (!c || !m || !weights_dev || !model_ok(m, n_floats)) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipStreamSynchronize(c->stream));
  vfk_free_model(c);
  c->has_model = false;
  c->model = *m;
  int rc = vfk_pack_model(c, weights_dev);
  if (rc != VF_OK) {
    vfk_free_model(c);
    return rc;
  }
  VF_HIP(c, hipStreamSynchronize(c->stream));  // weights_dev is not needed after return
  c->has_model = true;
  return VF_OK;
}

int vf_reset_state(vf_ctx *c) {
  if (!c) return VF_EINVAL;
  if (!c->has_pipeline) return VF_ESTATE;
  DeviceGuard g(c->device);
  c->n_sched = 0;
  c->seq_stage = -1;
  ++c->state_epoch;
  return vfk_reset_state(c);
}

int vf_set_state(vf_ctx *c, const int32_t *cids, int n) {
  if (!c || n < 0 || (n > 0 && !cids)) return VF_EINVAL;
  if (!c->has_pipeline) return VF_ESTATE;
  if (n > c->S) return VF_EINVAL;
  DeviceGuard g(c->device);
  int rc = vf_reset_state(c);
  if (rc != VF_OK || n == 0) return rc;
  // stage the ids as [B][S]
  std::vector<int32_t> tmp((size_t)c->B * c->S, -1);
  for (int b = 0; b < c->B; ++b)
    for (int j = 0; j < n; ++j) tmp[(size_t)b * c->S + j] = cids[(size_t)b * n + j];
  VF_HIP(c, hipMemcpyAsync(c->d_forced, tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice, c->stream));
  VF_HIP(c, hipStreamSynchronize(c->stream));
  for (int j = 0; j < n; ++j) {
    rc = vfk_commit_forced(c, j);
    if (rc != VF_OK) return rc;
  }
  int32_t err = 0;
  VF_HIP(c, hipMemcpyAsync(&err, c->d_err, 4, hipMemcpyDeviceToHost, c->stream));
  VF_HIP(c, hipStreamSynchronize(c->stream));
  if (err) {
    vf_reset_state(c);
    return VF_ESTATE;
  }
  c->n_sched = n;
  return VF_OK;
}

int vf_n_scheduled(const vf_ctx *c) { return c ? c->n_sched : 0; }
int64_t vf_dense_count(const vf_ctx *c) { return (c && c->has_space) ? c->M : 0; }
int64_t vf_padded_count(const vf_ctx *c) { return (c && c->has_space) ? c->Mpad : 0; }

int vf_enumerate(vf_ctx *c, int stage, uint32_t *dec, uint8_t *valid, int32_t *n_valid) {
  if (!c) return VF_EINVAL;
  if (!c->has_pipeline) return VF_ESTATE;
  if (stage < 0 || stage >= c->S) return VF_EINVAL;
  if (stage > c->n_sched) return VF_ESTATE;
  DeviceGuard g(c->device);
  const int rc = settle_whole(c, stage > 0);
  if (rc != VF_OK) return rc;
  return vfk_enumerate(c, stage, dec, valid, n_valid);
}

int vf_featurize(vf_ctx *c, int stage, int32_t *feat) {
  if (!c || !feat) return VF_EINVAL;
  if (!c->has_pipeline) return VF_ESTATE;
  if (stage < 0 || stage >= c->S) return VF_EINVAL;
  if (stage > c->n_sched) return VF_ESTATE;
  DeviceGuard g(c->device);
  const int rc = settle_whole(c, stage > 0);
  if (rc != VF_OK) return rc;
  return vfk_featurize(c, stage, feat);
}

// V(s) and the scan for given inputs.  parts == nullptr: the context's own growable buffers
// hold the per-workgroup minima (vf_score); otherwise the given buffer does and nothing is
// allocated (vf_score_static).
static int score_call(vf_ctx *c, const void *x, int32_t x_kind, int64_t M, int64_t ld, int32_t group, float *scores,
                      int32_t *best_idx, float *best_val, const vf_partbuf *parts) {
  const bool want_min = best_idx || best_val;
  int nparts = 0, part = 0, rc;
  if (x_kind == VF_X_RAW_I32) {
    if (c->model.kind != VF_MLP || ld < M) return VF_EINVAL;
    rc = vfk_score_mlp(c, (const int32_t *)x, 0, 1, M, ld, 0, scores, ld, &nparts, -1, parts);
    int maxw = 0;
    for (int l = 0; l < c->model.n_layers; ++l)
      if (c->model.dims[l] > maxw) maxw = c->model.dims[l];
    part = (c->model.dtype == VF_FP32) ? VF_PART : (maxw > 512 ? 64 : 128);
  } else if (x_kind == VF_X_SEQ_BF16) {
    if (c->model.kind != VF_LSTM || ld < 0 || ld > (1 << 20)) return VF_EINVAL;
    rc = vfk_score_lstm(c, (const uint16_t *)x, M, (int)ld, scores, &nparts, parts);
    part = 64;
  } else {
    return VF_EINVAL;
  }
  if (rc != VF_OK || !want_min) return rc;
  int64_t gsz = group > 0 ? group : (M > 0 ? M : 1);
  int ngroups = (int)((M + gsz - 1) / gsz);
  if (ngroups < 1) ngroups = 1;
  int ppg = (int)((gsz + part - 1) / part);
  if (!parts) {
    rc = vfk_ensure_parts(c, 1);
    if (rc != VF_OK) return rc;
  }
  return vfk_argmin_groups(c, M, nparts, ppg, ngroups, best_idx, best_val, parts);
}

int vf_score(vf_ctx *c, const void *x, int32_t x_kind, int64_t M, int64_t ld, int32_t group, float *scores,
             int32_t *best_idx, float *best_val) {
  if (!c || M < 0 || group < 0 || (M > 0 && !x)) return VF_EINVAL;
  if (!c->has_model) return VF_ESTATE;
  if (M > (int64_t)1 << 30) return VF_EINVAL;
  if ((best_idx || best_val) && group > 0 && group % 128 != 0) return VF_EINVAL;
  DeviceGuard g(c->device);
  return score_call(c, x, x_kind, M, ld, group, scores, best_idx, best_val, nullptr);
}

int vf_score_static(vf_ctx *c, const void *x, int32_t x_kind, int64_t M, int64_t ld, int32_t group, float *scores,
                    int32_t *best_idx, float *best_val) {
  if (!c || M < 0 || group < 0 || (M > 0 && !x)) return VF_EINVAL;
  if (!c->has_model) return VF_ESTATE;
  if (c->model.dtype != VF_BF16) return VF_EINVAL;  // the fp32 kernels keep activation matrices in scratch
  if (M > vf_score_static_max(c)) return VF_EINVAL;
  if ((best_idx || best_val) && group > 0 && group % 128 != 0) return VF_EINVAL;
  DeviceGuard g(c->device);
  if (!c->static_parts.val) return VF_ESTATE;
  const vf_partbuf parts = c->static_parts;
  int rc;
  // (event pairs of the per-kernel timing are created on demand: not in this call)
  const bool prof = c->profiling;
  c->profiling = false;
  rc = score_call(c, x, x_kind, M, ld, group, scores, best_idx, best_val, &parts);
  c->profiling = prof;
  return rc;
}

int64_t vf_score_static_max(const vf_ctx *c) {
  if (!c || !c->has_model || c->model.dtype != VF_BF16) return 0;
  int maxw = 0;
  if (c->model.kind == VF_MLP)
    for (int l = 0; l < c->model.n_layers; ++l)
      if (c->model.dims[l] > maxw) maxw = c->model.dims[l];
  const int64_t tile = (c->model.kind == VF_LSTM || maxw > 512) ? 64 : 128;  // candidates per workgroup
  return tile * VF_STATIC_PARTS;
}

int vf_argmin_step(vf_ctx *c, int stage, int commit, int32_t *best_cid, float *best_val) {
  if (!c) return VF_EINVAL;
  if (!c->has_pipeline || !c->has_model) return VF_ESTATE;
  if (!model_fits(c)) return VF_EINVAL;
  if (stage < 0 || stage >= c->S) return VF_EINVAL;
  if (stage != c->n_sched) return VF_ESTATE;
  DeviceGuard g(c->device);
  int rc = settle_whole(c, stage > 0);
  if (rc != VF_OK) return rc;
  rc = step(c, stage, commit, best_cid, best_val);
  if (rc == VF_OK && commit) c->n_sched = stage + 1;
  return rc;
}

int vf_greedy_schedule(vf_ctx *c, int first, int last, vf_state *out_states, int32_t *out_cids, float *out_vals) {
  if (!c) return VF_EINVAL;
  if (!c->has_pipeline || !c->has_model) return VF_ESTATE;
  if (!model_fits(c)) return VF_EINVAL;
  if (first < 0 || last >= c->S || first > last + 1) return VF_EINVAL;
  if (first != c->n_sched) return VF_ESTATE;
  DeviceGuard g(c->device);
  {
    // an earlier whole-schedule launch that gave up a wait: this call builds on its tables
    // unless it starts from s_0, so it waits for that launch's verdict; from s_0 it only
    // looks whether the verdict is in
    const int rc = settle_whole(c, first > 0);
    if (rc != VF_OK) return rc;
  }
  if (first <= last && vfk_whole_team(c) >= 1) {
    int rc = vfk_greedy_whole(c, first, last);
    if (rc != VF_OK) return rc;
    c->n_sched = last + 1;
  } else if (first <= last && vfk_can_chain(c)) {
    // a few problems: one launch per layer, each taking the decision of the layer before
    int rc = vfk_greedy_chain(c, first, last);
    if (rc != VF_OK) return rc;
    c->n_sched = last + 1;
  } else {
    for (int i = first; i <= last; ++i) {
      int rc = step(c, i, 1, nullptr, nullptr);
      if (rc != VF_OK) return rc;
      c->n_sched = i + 1;
    }
  }
  const size_t n = (size_t)c->B * c->S;
  if (out_states)
    VF_HIP(c, hipMemcpyAsync(out_states, c->d_states, n * sizeof(vf_state), hipMemcpyDeviceToDevice, c->stream));
  if (out_cids) VF_HIP(c, hipMemcpyAsync(out_cids, c->d_cids, n * 4, hipMemcpyDeviceToDevice, c->stream));
  if (out_vals) VF_HIP(c, hipMemcpyAsync(out_vals, c->d_vals, n * 4, hipMemcpyDeviceToDevice, c->stream));
  return VF_OK;
}

int vf_set_noise(vf_ctx *c, float eps, uint64_t seed, int32_t first_rollout) {
  if (!c || !(eps >= 0.0f) || eps > 3.0e38f || first_rollout < 0) return VF_EINVAL;
  c->noise_eps = eps;
  c->noise_seed = seed;
  c->noise_first = first_rollout;
  return VF_OK;
}

int vf_beam_search(vf_ctx *c, int first, int last, vf_state *out_states, int32_t *out_cids, float *out_vals,
                   int32_t *n_beams) {
  if (!c) return VF_EINVAL;
  if (!c->has_pipeline || !c->has_model) return VF_ESTATE;
  if (!model_fits(c)) return VF_EINVAL;
  if (first < 0 || last >= c->S || first > last + 1) return VF_EINVAL;
  if (first != c->n_sched) return VF_ESTATE;
  if ((int64_t)c->B * c->Mpad >= ((int64_t)1 << 31) || c->B > 1024) return VF_EINVAL;  // a selection pass keeps B of 2048
  if (!c->beam_checked) {
    for (int b = 1; b < c->B; ++b)
      if (memcmp(c->h_stages.data(), c->h_stages.data() + (size_t)b * c->S, sizeof(vf_stage) * (size_t)c->S) != 0)
        return VF_EINVAL;  // the slots of a beam search hold one and the same network
    c->beam_checked = true;
  }
  DeviceGuard g(c->device);
  int rc = settle_whole(c, first > 0);
  if (rc != VF_OK) return rc;
  rc = vfk_beam_init(c, first);
  if (rc != VF_OK) return rc;
  for (int i = first; i <= last; ++i) {
    rc = vfk_step_scores(c, i);
    if (rc != VF_OK) return rc;
    rc = vfk_beam_select_commit(c, i);
    if (rc != VF_OK) return rc;
    if (vfk_seq_model(c)) {
      rc = vfk_seq_advance_beam(c, i);  // survivors continue their parent's recurrence
      if (rc != VF_OK) return rc;
    }
    c->n_sched = i + 1;
  }
  const size_t n = (size_t)c->B * c->S;
  if (out_states)
    VF_HIP(c, hipMemcpyAsync(out_states, c->d_states, n * sizeof(vf_state), hipMemcpyDeviceToDevice, c->stream));
  if (out_cids) VF_HIP(c, hipMemcpyAsync(out_cids, c->d_cids, n * 4, hipMemcpyDeviceToDevice, c->stream));
  if (out_vals) VF_HIP(c, hipMemcpyAsync(out_vals, c->d_vals, n * 4, hipMemcpyDeviceToDevice, c->stream));
  if (n_beams) VF_HIP(c, hipMemcpyAsync(n_beams, c->d_sel_n + 1, 4, hipMemcpyDeviceToDevice, c->stream));
  return VF_OK;
}

const char *vf_strerror(int code) {
  switch (code) {
    case VF_OK: return "ok";
    case VF_EINVAL: return "invalid argument";
    case VF_ESTATE: return "call out of order or invalid scheduling state";
    case VF_ENOMEM: return "out of memory";
    case VF_EHIP: return "HIP runtime error (see vf_last_hip_error)";
    default: return "unknown error";
  }
}

int vf_last_hip_error(const vf_ctx *c) { return c ? c->last_hip : 0; }

int vf_timer_start(vf_ctx *c) {
  if (!c) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipEventRecord(c->ev0, c->stream));
  return VF_OK;
}
int vf_timer_stop(vf_ctx *c) {
  if (!c) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipEventRecord(c->ev1, c->stream));
  return VF_OK;
}
int vf_timer_elapsed_ms(vf_ctx *c, float *ms) {
  if (!c || !ms) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipEventSynchronize(c->ev1));
  VF_HIP(c, hipEventElapsedTime(ms, c->ev0, c->ev1));
  return VF_OK;
}

int vf_profile_enable(vf_ctx *c, int enable) {
  if (!c) return VF_EINVAL;
  c->profiling = enable != 0;
  return VF_OK;
}

int vf_profile_read(vf_ctx *c, int which, double *total_ms, int64_t *launches) {
  if (!c || which < 0 || which > 2) return VF_EINVAL;
  DeviceGuard g(c->device);
  auto &v = c->prof_pairs[which];
  double sum = 0.0;
  for (size_t k = 0; k + 1 < v.size(); k += 2) {
    VF_HIP(c, hipEventSynchronize(v[k + 1]));
    float ms = 0.0f;
    VF_HIP(c, hipEventElapsedTime(&ms, v[k], v[k + 1]));
    sum += ms;
  }
  if (total_ms) *total_ms = sum;
  if (launches) *launches = (int64_t)(v.size() / 2);
  for (hipEvent_t e : v) c->prof_free.push_back(e);
  v.clear();
  return VF_OK;
}

int vf_profile_counts(vf_ctx *c, int64_t *scored, int64_t *valid) {
  if (!c) return VF_EINVAL;
  DeviceGuard g(c->device);
  unsigned long long h[2] = {0ull, 0ull};
  VF_HIP(c, hipMemcpyAsync(h, c->d_stat, 16, hipMemcpyDeviceToHost, c->stream));
  VF_HIP(c, hipMemsetAsync(c->d_stat, 0, 16, c->stream));
  VF_HIP(c, hipStreamSynchronize(c->stream));
  if (scored) *scored = (int64_t)h[0];
  if (valid) *valid = (int64_t)h[1];
  return VF_OK;
}

int vf_sync_status(vf_ctx *c) {
  if (!c) return VF_EINVAL;
  DeviceGuard g(c->device);
  VF_HIP(c, hipStreamSynchronize(c->stream));
  const int rc = settle_whole(c, true);
  if (rc == VF_ESTATE) VF_HIP(c, hipStreamSynchronize(c->stream));  // the repair, if any, has run as well
  return rc;
}

int vf_set_wait_limit(vf_ctx *c, unsigned int rounds) {
  if (!c) return VF_EINVAL;
  c->wait_rounds = rounds;
  return VF_OK;
}

}  // extern "C"
