/*
 * CPU checker for the value-function-guided greedy scheduler of
 * "Value Function Based Performance Optimization of Deep Learning Workloads"
 * (Steiner, Cummins, He, Leather; arXiv 2011.14486).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar implementation
 * used to check the GPU library and to provide a timed CPU baseline.  It shares no
 * code, header, table or helper with the GPU library and must never be called from
 * the product path.
 *
 * What it follows:
 *   - Algorithm 1 ("Scheduling"): for each layer in order, scan the candidate
 *     states, keep the first one whose value is strictly smaller than the
 *     incumbent (v_i starts at +infinity), commit it, go on to the next layer.
 *   - Section 2 (MDP formulation): a state is the set of decisions for the layers
 *     scheduled so far; the options for the next layer depend on the loop
 *     structure those decisions impose.
 *   - Table 1: a candidate is one choice for each of split, reorder, vectorize,
 *     parallel, compute_at and store_at.
 *   - Section 3.2 ("Implementation"): schedule-invariant ("intrinsic") and
 *     schedule-dependent ("acquired") features, normalised, fed to the value
 *     network; the recurrent network's per-timestep predictions are summed.
 *
 * The paper names the kinds of features and actions but lists neither, and gives no
 * network sizes.  The concrete candidate space, validity rules, the 64 / 256 feature
 * layout, the piecewise-linear log2 normalisation and the MLP stand-in for V are
 * this project's reading of those passages; they are written out in the project's
 * design notes and implemented here directly from that prose.  Nothing in the paper
 * can confirm that reading ("parity unpinned" against the paper for the feature list
 * and the candidate space); every function below is pinned by closed forms,
 * invariants, brute force or a library routine in the CPU tests.
 *
 * Conventions: all feature arithmetic is on non-negative integers and saturates at
 * 2^31-1; no floating point is used before the normalisation step.  Network
 * arithmetic accumulates in double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { K_CONV = 0, K_DWCONV = 1, K_POINTWISE = 2, K_ADD = 3 };
enum { AT_ROOT = 0, AT_L1 = 1, AT_L2 = 2, AT_INLINE = 3 };
enum { OVF_OK = 0, OVF_EINVAL = -1, OVF_ESTATE = -2, OVF_ENOMEM = -3 };

typedef struct { int32_t w[16]; } ovf_stage;
typedef struct { int32_t w[16]; } ovf_state;
typedef struct {
  int32_t nf[3];
  int32_t fac[3][8];
  int32_t nperm;
  int32_t perm[8][3];
  int32_t nvec, npar, ncat;
  int32_t cat[4];
  int32_t nsat;
  int32_t vlen, ncores, l1_bytes, l2_bytes, F;
} ovf_space;
typedef struct { int32_t kind, n_layers, dims[8], dtype; } ovf_model;

/* optional user-supplied value function (used by the exact-V test):
 * core64 = the 64 core features of the candidate state */
typedef double (*ovf_vfun)(void *user, int32_t stage, int32_t cid, const int32_t *core64);

/* ---------------------------------------------------------------- integers */

#define SATMAX 2147483647LL

static int64_t satmul(int64_t a, int64_t b) {
  uint64_t p = (uint64_t)a * (uint64_t)b; /* both < 2^31, no overflow */
  return p > (uint64_t)SATMAX ? SATMAX : (int64_t)p;
}
static int64_t satadd(int64_t a, int64_t b) {
  int64_t s = a + b;
  return s > SATMAX ? SATMAX : s;
}
static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }
static int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
/* fixed-point ratio with 4 fractional bits */
static int64_t ratio16(int64_t num, int64_t den) { return satmul(num, 16) / max64(den, 1); }

int64_t ovf_dense_count(const ovf_space *sp) {
  int64_t m = 1;
  m *= sp->nf[0]; m *= sp->nf[1]; m *= sp->nf[2];
  m *= sp->nperm; m *= sp->nvec; m *= sp->npar; m *= sp->ncat; m *= sp->nsat;
  return m;
}

int64_t ovf_padded_count(const ovf_space *sp) {
  return (ovf_dense_count(sp) + 255) / 256 * 256;
}

static int space_ok(const ovf_space *sp) {
  for (int d = 0; d < 3; ++d) {
    if (sp->nf[d] < 1 || sp->nf[d] > 8) return 0;
    for (int k = 0; k < sp->nf[d]; ++k) if (sp->fac[d][k] < 1) return 0;
  }
  if (sp->nperm < 1 || sp->nperm > 8) return 0;
  for (int p = 0; p < sp->nperm; ++p) {
    int seen = 0;
    for (int k = 0; k < 3; ++k) {
      if (sp->perm[p][k] < 0 || sp->perm[p][k] > 2) return 0;
      seen |= 1 << sp->perm[p][k];
    }
    if (seen != 7) return 0;
  }
  if (sp->nvec < 1 || sp->nvec > 2 || sp->npar < 1 || sp->npar > 2) return 0;
  if (sp->ncat < 1 || sp->ncat > 4) return 0;
  for (int k = 0; k < sp->ncat; ++k) if (sp->cat[k] < 0 || sp->cat[k] > 3) return 0;
  if (sp->nsat < 1 || sp->nsat > 3) return 0;
  if (sp->vlen < 1 || sp->ncores < 1 || sp->l1_bytes < 0 || sp->l2_bytes < 0) return 0;
  if (sp->F != 64 && sp->F != 256) return 0;
  if (ovf_dense_count(sp) > (1 << 30)) return 0;
  return 1;
}

static int pipeline_ok(const ovf_stage *st, int S) {
  if (S < 1) return 0;
  for (int j = 0; j < S; ++j) {
    const int32_t *w = st[j].w;
    if (w[0] < 0 || w[0] > 3) return 0;
    for (int k = 1; k <= 7; ++k) if (w[k] < 1) return 0;
    if (w[8] < -1 || w[8] >= j) return 0; /* the anchor is listed earlier */
    if (w[9] < 0 || w[12] < 1) return 0;
  }
  return 1;
}

/* ------------------------------------------- intrinsic (schedule-invariant) */

/* Section 3.2: amount of computation and data access of stage j, independent of
 * any schedule.  a[0..15] is feature block A. */
static void intrinsic(const ovf_stage *stages, int S, int j, int32_t a[16]) {
  const int32_t *w = stages[j].w;
  int64_t kind = w[0], W = w[1], H = w[2], C = w[3], RC = w[4], KH = w[5], KW = w[6];
  int64_t stride = w[7], eb = w[12];
  int64_t R = satmul(satmul(RC, KH), KW);
  int64_t points = satmul(satmul(W, H), C);
  int64_t macs = (kind == K_CONV || kind == K_DWCONV) ? satmul(points, R) : points;
  int64_t cin = (kind == K_CONV) ? RC : C;
  int64_t in_elems = satmul(satmul(satmul(W, stride), satmul(H, stride)), cin);
  if (kind == K_ADD) in_elems = satmul(in_elems, 2);
  int64_t w_elems = 0;
  if (kind == K_CONV) w_elems = satmul(satmul(satmul(C, RC), KH), KW);
  if (kind == K_DWCONV) w_elems = satmul(satmul(C, KH), KW);
  a[0] = (int32_t)kind;
  a[1] = (int32_t)W; a[2] = (int32_t)H; a[3] = (int32_t)C;
  a[4] = (int32_t)R;
  a[5] = (int32_t)satmul(KH, KW);
  a[6] = (int32_t)stride;
  a[7] = (int32_t)points;
  a[8] = (int32_t)macs;
  a[9] = (int32_t)in_elems;
  a[10] = (int32_t)w_elems;
  a[11] = (int32_t)satmul(points, eb);
  a[12] = (int32_t)ratio16(macs, satadd(satadd(in_elems, w_elems), points));
  a[13] = w[9];
  a[14] = j;
  a[15] = S - 1 - j;
}

/* --------------------------------------------------- region of a producer */

/* Part of stage i's output that one instance of its loop nest must produce when
 * it is computed at `level` of its anchor's loop nest, and how many instances run.
 * srec = stage i, arec/ast = anchor's record and committed state. */
static void region_at(int level, const int32_t *srec, const int32_t *arec,
                      const ovf_state *ast, const ovf_space *sp, int64_t E[3], int64_t *inst) {
  int64_t ext[3] = { srec[1], srec[2], srec[3] };
  if (level == AT_ROOT) {
    E[0] = ext[0]; E[1] = ext[1]; E[2] = ext[2];
    *inst = 1;
    return;
  }
  int64_t fa[3] = { ast->w[0], ast->w[1], ast->w[2] };
  int64_t Ea[3] = { ast->w[8], ast->w[9], ast->w[10] };
  int64_t Oa[3] = { ast->w[12], ast->w[13], ast->w[14] };
  int64_t inst_a = ast->w[11];
  int64_t box[3];
  if (level == AT_L1) {
    int d0 = sp->perm[ast->w[3]][0];
    box[0] = Ea[0]; box[1] = Ea[1]; box[2] = Ea[2];
    box[d0] = fa[d0];
    *inst = satmul(inst_a, Oa[d0]);
  } else { /* AT_L2 */
    box[0] = fa[0]; box[1] = fa[1]; box[2] = fa[2];
    *inst = satmul(inst_a, satmul(satmul(Oa[0], Oa[1]), Oa[2]));
  }
  int64_t stride_a = arec[7], KH_a = arec[5], KW_a = arec[6];
  E[0] = min64(ext[0], satadd(satmul(box[0] - 1, stride_a), KW_a));
  E[1] = min64(ext[1], satadd(satmul(box[1] - 1, stride_a), KH_a));
  E[2] = (arec[0] == K_CONV) ? ext[2] : min64(ext[2], box[2]);
}

/* ------------------------------------------------------------ one candidate */

typedef struct {
  const ovf_stage *stages;
  int S;
  const ovf_space *sp;
  int i;                /* stage being decided; stages 0..i-1 are committed */
  const ovf_state *st;  /* [i] committed state records */
  const int32_t *cf;    /* [i][64] committed core feature vectors */
} decision;

/* Decode candidate `cid` of decision d (Table 1: one choice per primitive), test
 * it against the loop structure of the committed stages, and compute its 64 core
 * features and the state record it would commit.  Returns the validity flag. */
static int candidate(const decision *d, int64_t cid, uint32_t *dec_out,
                     int32_t core[64], ovf_state *state_out) {
  const ovf_space *sp = d->sp;
  const int32_t *srec = d->stages[d->i].w;
  const int i = d->i;

  /* mixed-radix digits, least significant first */
  int64_t r = cid;
  int ix = (int)(r % sp->nf[0]); r /= sp->nf[0];
  int iy = (int)(r % sp->nf[1]); r /= sp->nf[1];
  int ic = (int)(r % sp->nf[2]); r /= sp->nf[2];
  int ip = (int)(r % sp->nperm); r /= sp->nperm;
  int vec = (int)(r % sp->nvec); r /= sp->nvec;
  int par = (int)(r % sp->npar); r /= sp->npar;
  int icat = (int)(r % sp->ncat); r /= sp->ncat;
  int isat = (int)r;
  if (dec_out)
    *dec_out = (uint32_t)ix | (uint32_t)iy << 4 | (uint32_t)ic << 8 | (uint32_t)ip << 12 |
               (uint32_t)vec << 16 | (uint32_t)par << 20 | (uint32_t)icat << 24 | (uint32_t)isat << 28;

  int cat = sp->cat[icat];
  int hoist = isat;
  int64_t f[3] = { sp->fac[0][ix], sp->fac[1][iy], sp->fac[2][ic] };

  for (int k = 0; k < 64; ++k) core[k] = 0;
  intrinsic(d->stages, d->S, i, core); /* block A is written for every candidate */
  if (state_out) memset(state_out, 0, sizeof *state_out);

  const int kind = srec[0];
  const int a = srec[8];
  const int anchored = (a >= 0 && a < i && d->st[a].w[15] == 1);
  const int32_t *arec = anchored ? d->stages[a].w : NULL;
  const ovf_state *ast = anchored ? &d->st[a] : NULL;

  /* --- validity (the dynamic action space of Section 2) --- */
  int valid = 1;
  if (cat != AT_ROOT) {
    if (!(anchored && srec[9] == 1)) valid = 0;
  }
  if (valid && (cat == AT_L1 || cat == AT_L2)) {
    if (ast->w[6] == AT_INLINE) valid = 0;
    else if (cat == AT_L1) {
      int d0 = sp->perm[ast->w[3]][0];
      if (!(ast->w[12 + d0] > 1)) valid = 0;
    } else {
      int64_t tiles = satmul(satmul(ast->w[12], ast->w[13]), ast->w[14]);
      if (!(tiles > 1)) valid = 0;
    }
  }
  if (valid && cat == AT_INLINE) {
    if (!(kind == K_POINTWISE || kind == K_ADD)) valid = 0;
    if (ix || iy || ic || ip || vec || par || isat) valid = 0;
  }
  if (valid && cat != AT_INLINE && hoist > cat) valid = 0;

  int64_t E[3] = { 1, 1, 1 }, inst = 1;
  if (valid) {
    if (cat == AT_INLINE) {
      f[0] = f[1] = f[2] = 1;
      int64_t pp = 1;
      for (int k = 0; k < 3; ++k) pp = satmul(satmul(pp, ast->w[12 + k]), ast->w[k]);
      int64_t Ra = satmul(satmul(arec[4], arec[5]), arec[6]);
      inst = satmul(satmul(ast->w[11], pp), Ra);
    } else {
      region_at(cat, srec, arec, ast, sp, E, &inst);
      for (int k = 0; k < 3; ++k)
        if (f[k] > E[k]) valid = 0; /* a factor larger than the loop is not a split */
    }
  }
  if (!valid) return 0;

  /* --- acquired features (block B) --- */
  const int32_t *pi = sp->perm[ip];
  int64_t O[3];
  for (int k = 0; k < 3; ++k) O[k] = ceil_div(E[k], f[k]);
  int64_t R = core[4];
  int64_t eb = srec[12], stride = srec[7], KH = srec[5], KW = srec[6], RC = srec[4];

  core[16] = 1;
  core[17] = (int32_t)f[0]; core[18] = (int32_t)f[1]; core[19] = (int32_t)f[2];
  core[20] = (int32_t)O[0]; core[21] = (int32_t)O[1]; core[22] = (int32_t)O[2];
  core[23] = ip;
  core[24] = pi[2];
  core[25] = pi[0];
  core[26] = vec;
  int64_t fin = f[pi[2]];
  core[27] = (int32_t)(vec ? min64(fin, sp->vlen) : 1);
  core[28] = (int32_t)(vec ? ratio16(fin, satmul(ceil_div(fin, sp->vlen), sp->vlen)) : 16);
  core[29] = par;
  int64_t tasks = par ? O[pi[0]] : 1;
  core[30] = (int32_t)tasks;
  core[31] = (int32_t)ratio16(tasks, satmul(ceil_div(tasks, sp->ncores), sp->ncores));
  core[32] = cat;
  core[33] = hoist;
  core[34] = (int32_t)E[0]; core[35] = (int32_t)E[1]; core[36] = (int32_t)E[2];
  core[37] = (int32_t)inst;
  int64_t padded = 1;
  for (int k = 0; k < 3; ++k) padded = satmul(satmul(padded, O[k]), f[k]);
  core[38] = (int32_t)padded;
  int64_t total_points = satmul(inst, padded);
  core[39] = (int32_t)total_points;
  core[40] = (int32_t)satmul(total_points, R);
  core[41] = (int32_t)ratio16(total_points, core[7]);
  int64_t tile_points = satmul(satmul(f[0], f[1]), f[2]);
  core[42] = (int32_t)tile_points;
  int64_t tin = satmul(satadd(satmul(f[0] - 1, stride), KW), satadd(satmul(f[1] - 1, stride), KH));
  tin = satmul(tin, kind == K_CONV ? RC : f[2]);
  if (kind == K_ADD) tin = satmul(tin, 2);
  core[43] = (int32_t)tin;
  int64_t tw = 0;
  if (kind == K_CONV) tw = satmul(satmul(satmul(f[2], RC), KH), KW);
  if (kind == K_DWCONV) tw = satmul(satmul(f[2], KH), KW);
  core[44] = (int32_t)tw;
  int64_t ws = satadd(satadd(tile_points, tin), tw);
  core[45] = (int32_t)ws;
  core[46] = satmul(ws, eb) <= sp->l1_bytes;
  core[47] = satmul(ws, eb) <= sp->l2_bytes;
  if (cat == AT_INLINE) {
    core[48] = 0;
    core[49] = 0;
  } else {
    int64_t Es[3], insts;
    region_at(cat - hoist, srec, arec, ast, sp, Es, &insts);
    core[48] = (int32_t)satmul(satmul(Es[0], Es[1]), Es[2]);
    core[49] = (int32_t)insts;
  }
  core[50] = (int32_t)(cat == AT_INLINE ? 0 : satmul(total_points, eb));
  int64_t ntiles = satmul(satmul(O[0], O[1]), O[2]);
  core[51] = (int32_t)satmul(satmul(inst, ntiles), satmul(satadd(tin, tw), eb));
  core[52] = (int32_t)(pi[2] == 0 ? f[0] : 1);
  core[53] = (int32_t)ratio16(satmul(tile_points, R), satadd(tin, tw));
  core[54] = (int32_t)ntiles;
  core[55] = (E[0] % f[0] == 0) && (E[1] % f[1] == 0) && (E[2] % f[2] == 0);

  /* --- context (block C): what the schedule so far looks like --- */
  if (anchored) {
    const int32_t *ac = d->cf + 64 * (size_t)a;
    core[56] = ac[42];
    core[57] = ac[54];
    core[58] = ac[32];
    core[59] = (ip == ac[23]);
  }
  int64_t pm = 0, pb = 0, sm = 0, spt = 0;
  for (int j = 0; j < i; ++j) {
    pm = satadd(pm, d->cf[64 * (size_t)j + 40]);
    pb = satadd(pb, d->cf[64 * (size_t)j + 50]);
  }
  for (int j = i + 1; j < d->S; ++j) {
    int32_t aj[16];
    intrinsic(d->stages, d->S, j, aj);
    sm = satadd(sm, aj[8]);
    spt = satadd(spt, aj[7]);
  }
  core[60] = (int32_t)pm; core[61] = (int32_t)pb; core[62] = (int32_t)sm; core[63] = (int32_t)spt;

  if (state_out) {
    int32_t *s = state_out->w;
    s[0] = (int32_t)f[0]; s[1] = (int32_t)f[1]; s[2] = (int32_t)f[2];
    s[3] = ip; s[4] = vec; s[5] = par; s[6] = cat; s[7] = hoist;
    s[8] = (int32_t)E[0]; s[9] = (int32_t)E[1]; s[10] = (int32_t)E[2];
    s[11] = (int32_t)inst;
    s[12] = (int32_t)O[0]; s[13] = (int32_t)O[1]; s[14] = (int32_t)O[2];
    s[15] = 1;
  }
  return 1;
}

/* Replay the committed prefix: state records and core features of stages
 * 0..n-1 given the candidate ids chosen for them.  OVF_ESTATE if one of them is
 * not a valid candidate. */
static int replay(const ovf_stage *stages, int S, const ovf_space *sp, const int32_t *cids,
                  int n, ovf_state *st, int32_t *cf) {
  int64_t M = ovf_dense_count(sp);
  for (int j = 0; j < n; ++j) {
    if (cids[j] < 0 || cids[j] >= M) return OVF_ESTATE;
    decision d = { stages, S, sp, j, st, cf };
    if (!candidate(&d, cids[j], NULL, cf + 64 * (size_t)j, &st[j])) return OVF_ESTATE;
  }
  return OVF_OK;
}

/* State records of a committed prefix. */
int ovf_states(const ovf_stage *stages, int S, const ovf_space *sp, const int32_t *cids,
               int n, ovf_state *out, int32_t *core_out /* nullable, [n][64] */) {
  if (!space_ok(sp) || !pipeline_ok(stages, S) || n < 0 || n > S) return OVF_EINVAL;
  int32_t *cf = (int32_t *)calloc((size_t)(n > 0 ? n : 1) * 64, sizeof(int32_t));
  if (!cf) return OVF_ENOMEM;
  int rc = replay(stages, S, sp, cids, n, out, cf);
  if (rc == OVF_OK && core_out) memcpy(core_out, cf, (size_t)n * 64 * sizeof(int32_t));
  free(cf);
  return rc;
}

/* C_i = CandidateActions(L_i, s_{i-1}) of Algorithm 1 as a dense id range with a
 * validity flag.  dec/valid have M_pad entries; padding entries are zero. */
int ovf_enumerate(const ovf_stage *stages, int S, const ovf_space *sp, const int32_t *prefix_cids,
                  int stage, uint32_t *dec, uint8_t *valid, int32_t *n_valid) {
  if (!space_ok(sp) || !pipeline_ok(stages, S) || stage < 0 || stage >= S) return OVF_EINVAL;
  int64_t M = ovf_dense_count(sp), Mp = ovf_padded_count(sp);
  int n = stage > 0 ? stage : 1;
  ovf_state *st = (ovf_state *)calloc((size_t)n, sizeof(ovf_state));
  int32_t *cf = (int32_t *)calloc((size_t)n * 64, sizeof(int32_t));
  if (!st || !cf) { free(st); free(cf); return OVF_ENOMEM; }
  int rc = replay(stages, S, sp, prefix_cids, stage, st, cf);
  if (rc == OVF_OK) {
    decision d = { stages, S, sp, stage, st, cf };
    int32_t count = 0;
    for (int64_t cid = 0; cid < Mp; ++cid) {
      if (cid >= M) { dec[cid] = 0; valid[cid] = 0; continue; }
      int32_t core[64];
      int v = candidate(&d, cid, &dec[cid], core, NULL);
      valid[cid] = (uint8_t)v;
      count += v;
    }
    *n_valid = count;
  }
  free(st); free(cf);
  return rc;
}

/* Features of every candidate state of decision `stage`: feat[f*M_pad + cid],
 * F rows.  Rows 0..63 are the core vector.  With F = 256, rows 64..207 are
 * features 0..47 of the committed vectors of stages i-1, i-2, i-3 and rows 208..255
 * are block A of stages i+1, i+2, i+3 (zero where there is no such stage).  Invalid
 * candidates keep block A and the neighbour rows, their rows 16..63 are zero.
 * Padding columns are zero. */
int ovf_featurize(const ovf_stage *stages, int S, const ovf_space *sp, const int32_t *prefix_cids,
                  int stage, int32_t *feat) {
  if (!space_ok(sp) || !pipeline_ok(stages, S) || stage < 0 || stage >= S) return OVF_EINVAL;
  int64_t M = ovf_dense_count(sp), Mp = ovf_padded_count(sp);
  int F = sp->F;
  int n = stage > 0 ? stage : 1;
  ovf_state *st = (ovf_state *)calloc((size_t)n, sizeof(ovf_state));
  int32_t *cf = (int32_t *)calloc((size_t)n * 64, sizeof(int32_t));
  if (!st || !cf) { free(st); free(cf); return OVF_ENOMEM; }
  int rc = replay(stages, S, sp, prefix_cids, stage, st, cf);
  if (rc == OVF_OK) {
    decision d = { stages, S, sp, stage, st, cf };
    int32_t nb[192];
    memset(nb, 0, sizeof nb);
    for (int k = 1; k <= 3; ++k) {
      if (stage - k >= 0)
        for (int t = 0; t < 48; ++t) nb[48 * (k - 1) + t] = cf[64 * (size_t)(stage - k) + t];
      if (stage + k < S) intrinsic(stages, S, stage + k, nb + 144 + 16 * (k - 1));
    }
    memset(feat, 0, (size_t)F * (size_t)Mp * sizeof(int32_t));
#pragma omp parallel for schedule(static)
    for (int64_t cid = 0; cid < M; ++cid) {
      int32_t core[64];
      candidate(&d, cid, NULL, core, NULL);
      for (int k = 0; k < 64; ++k) feat[(size_t)k * Mp + cid] = core[k];
      if (F == 256)
        for (int k = 0; k < 192; ++k) feat[(size_t)(64 + k) * Mp + cid] = nb[k];
    }
  }
  free(st); free(cf);
  return rc;
}

/* ------------------------------------------------------------ normalisation */

/* Piecewise-linear log2 of a non-negative integer (Section 3.2 only says the
 * features are normalised; this is the project's reading): 0 -> 0, otherwise
 * exponent + (significand - 1) of the value converted to float. */
float ovf_plog2(int32_t x) {
  if (x <= 0) return 0.0f;
  float xf = (float)x;          /* round to nearest even */
  int ex;
  float mant = frexpf(xf, &ex); /* xf = mant * 2^ex, mant in [0.5, 1) */
  float m = mant * 2.0f;        /* exact */
  return (float)(ex - 1) + (m - 1.0f);
}

/* float -> bfloat16 (upper 16 bits of the IEEE-754 binary32 pattern), round to
 * nearest, ties to even; returned widened back to float. */
static float bf16_round(float v) {
  uint32_t u;
  memcpy(&u, &v, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) { u |= 0x00400000u; u &= 0xffff0000u; }
  else {
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
  }
  float r;
  memcpy(&r, &u, 4);
  return r;
}
float ovf_bf16_round(float v) { return bf16_round(v); }

static float bf16_bits_to_float(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float r;
  memcpy(&r, &u, 4);
  return r;
}

/* ------------------------------------------------------------------- V(s) */

/* MLP value network on one normalised input vector x[F] (already rounded if the
 * model is bf16).  weights: W_1, b_1, ..., W_L, b_L, W_k[out][in].  bf16 model:
 * weights and every hidden activation are rounded to bf16; sums, bias adds and the
 * last layer stay unrounded.  Scratch h0/h1 hold max(dims) doubles each. */
static double mlp_eval(const ovf_model *m, const float *weights, const double *x,
                       double *h0, double *h1) {
  const int bf = (m->dtype == 1);
  const int L = m->n_layers;
  const float *p = weights;
  const double *in = x;
  double *out = h0;
  double v = 0.0;
  for (int k = 0; k < L; ++k) {
    int fin = m->dims[k], fout = m->dims[k + 1];
    const float *W = p, *b = p + (size_t)fin * fout;
    for (int o = 0; o < fout; ++o) {
      double acc = 0.0;
      for (int q = 0; q < fin; ++q) {
        float wv = W[(size_t)o * fin + q];
        if (bf) wv = bf16_round(wv);
        acc += (double)wv * in[q];
      }
      acc += (double)b[o];
      if (k < L - 1) {
        if (acc < 0.0) acc = 0.0; /* ReLU; NaN stays NaN */
        if (bf) acc = (double)bf16_round((float)acc);
        out[o] = acc;
      } else {
        v = acc; /* dims[L] == 1 */
      }
    }
    p = b + fout;
    in = out;
    out = (out == h0) ? h1 : h0;
  }
  return v;
}

static int mlp_ok(const ovf_model *m) {
  if (m->kind != 0 || m->n_layers < 1 || m->n_layers > 7) return 0;
  for (int k = 0; k <= m->n_layers; ++k) if (m->dims[k] < 1) return 0;
  if (m->dims[m->n_layers] != 1) return 0;
  if (m->dtype != 0 && m->dtype != 1) return 0;
  return 1;
}

static int max_dim(const ovf_model *m) {
  int mx = 1;
  for (int k = 0; k <= m->n_layers; ++k) if (m->dims[k] > mx) mx = m->dims[k];
  return mx;
}

/* Scores of M candidates from raw integer features x[f*ld + n], f < dims[0]. */
int ovf_score_mlp(const ovf_model *m, const float *weights, const int32_t *x, int64_t ld,
                  int64_t M, float *scores) {
  if (!mlp_ok(m) || M < 0 || ld < M) return OVF_EINVAL;
  const int F = m->dims[0], mx = max_dim(m);
  int fail = 0;
#pragma omp parallel
  {
    double *buf = (double *)malloc(sizeof(double) * (size_t)(F + 2 * mx));
    if (!buf) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t n = 0; n < M; ++n) {
      if (!buf) continue;
      for (int q = 0; q < F; ++q) {
        float v = ovf_plog2(x[(size_t)q * ld + n]);
        if (m->dtype == 1) v = bf16_round(v);
        buf[q] = (double)v;
      }
      scores[n] = (float)mlp_eval(m, weights, buf, buf + F, buf + F + mx);
    }
    free(buf);
  }
  return fail ? OVF_ENOMEM : OVF_OK;
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* Recurrent value network (Section 3.2): an LSTM walks the per-stage feature
 * sequence x[n][t][:] (bf16 bit patterns, already normalised); a linear head is
 * applied to every h_t and the T predictions are summed.
 * weights: W_ih[4H][F], W_hh[4H][H], b_ih[4H], b_hh[4H], w_head[H], b_head; gate
 * blocks in the order i, f, g, o.  bf16 model: the matrices, the head vector, x_t
 * and the h_{t-1} fed back into the recurrence are bf16; gates, cell state and the
 * head's sum are not rounded. */
int ovf_score_lstm(const ovf_model *m, const float *weights, const uint16_t *x, int64_t B,
                   int32_t T, float *scores) {
  if (m->kind != 1 || m->n_layers != 2 || m->dims[0] < 1 || m->dims[1] < 1 || m->dims[2] != 1)
    return OVF_EINVAL;
  if (m->dtype != 0 && m->dtype != 1) return OVF_EINVAL;
  if (B < 0 || T < 0) return OVF_EINVAL;
  const int F = m->dims[0], H = m->dims[1], bf = (m->dtype == 1);
  const float *Wih = weights, *Whh = Wih + (size_t)4 * H * F;
  const float *bih = Whh + (size_t)4 * H * H, *bhh = bih + 4 * H;
  const float *wh = bhh + 4 * H, *bh = wh + H;
  /* weights as the model sees them */
  size_t nw = (size_t)4 * H * F + (size_t)4 * H * H;
  float *Wr = (float *)malloc(sizeof(float) * (nw + (size_t)H));
  if (!Wr) return OVF_ENOMEM;
  for (size_t k = 0; k < nw; ++k) Wr[k] = bf ? bf16_round(Wih[k]) : Wih[k];
  for (int k = 0; k < H; ++k) Wr[nw + k] = bf ? bf16_round(wh[k]) : wh[k];
  const float *Wi = Wr, *Wh = Wr + (size_t)4 * H * F, *whr = Wr + nw;
  int fail = 0;
#pragma omp parallel
  {
    double *h = (double *)malloc(sizeof(double) * (size_t)(7 * H));
    if (!h) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t n = 0; n < B; ++n) {
      if (!h) continue;
      double *hfb = h + H, *c = h + 2 * H, *z = h + 3 * H; /* z: 4H pre-activations */
      for (int k = 0; k < H; ++k) { h[k] = 0.0; hfb[k] = 0.0; c[k] = 0.0; }
      double v = 0.0;
      for (int t = 0; t < T; ++t) {
        const uint16_t *xt = x + ((size_t)n * T + t) * F;
        for (int r = 0; r < 4 * H; ++r) {
          double acc = 0.0;
          for (int q = 0; q < F; ++q) acc += (double)Wi[(size_t)r * F + q] * (double)bf16_bits_to_float(xt[q]);
          acc += (double)bih[r];
          double acc2 = 0.0;
          for (int q = 0; q < H; ++q) acc2 += (double)Wh[(size_t)r * H + q] * hfb[q];
          z[r] = acc + acc2 + (double)bhh[r];
        }
        double pred = 0.0;
        for (int k = 0; k < H; ++k) {
          double ig = sigmoid(z[k]), fg = sigmoid(z[H + k]);
          double gg = tanh(z[2 * H + k]), og = sigmoid(z[3 * H + k]);
          c[k] = fg * c[k] + ig * gg;
          h[k] = og * tanh(c[k]);
          pred += (double)whr[k] * h[k];
        }
        v += pred + (double)bh[0];
        for (int k = 0; k < H; ++k) hfb[k] = bf ? (double)bf16_round((float)h[k]) : h[k];
      }
      scores[n] = (float)v;
    }
    free(h);
  }
  free(Wr);
  return fail ? OVF_ENOMEM : OVF_OK;
}

/* ------------------------------------------------- V(s) on a whole schedule */

static int lstm_ok(const ovf_model *m) {
  return m && m->kind == 1 && m->n_layers == 2 && m->dims[0] >= 1 && m->dims[1] >= 1 && m->dims[2] == 1 &&
         (m->dtype == 0 || m->dtype == 1);
}

static uint16_t bf16_bits_of(float v) {
  float r = bf16_round(v);
  uint32_t u;
  memcpy(&u, &r, 4);
  return (uint16_t)(u >> 16);
}

/* The state of Section 2 as the sequence the recurrent network of Section 3.2 reads:
 * one timestep per stage of the pipeline, in scheduling order, 64 values each.  A stage
 * that is scheduled in the state contributes its whole core vector (intrinsic and
 * acquired features); a stage that is not scheduled yet contributes its intrinsic block
 * (rows 0..15) and zeros.  For candidate `cid` of decision d: stages 0..i-1 give the
 * vectors stored when they were committed, stage i gives the candidate's vector,
 * stages i+1.. are unscheduled.  Values are normalised and rounded to bf16. */
static void sequence_of(const decision *d, const int32_t core[64], uint16_t *x /* [S][64] */) {
  for (int t = 0; t < d->S; ++t) {
    int32_t row[64];
    memset(row, 0, sizeof row);
    if (t < d->i) memcpy(row, d->cf + 64 * (size_t)t, sizeof row);
    else if (t == d->i) memcpy(row, core, sizeof row);
    else intrinsic(d->stages, d->S, t, row);
    for (int k = 0; k < 64; ++k) x[(size_t)t * 64 + k] = bf16_bits_of(ovf_plog2(row[k]));
  }
}

/* Sequences of every candidate state of decision `stage` (x[cid][t][k], M entries, not
 * padded) and their validity flags.  An invalid candidate's own timestep has zeros in
 * rows 16..63, like its feature column. */
int ovf_sequences(const ovf_stage *stages, int S, const ovf_space *sp, const int32_t *prefix_cids,
                  int stage, uint16_t *x, uint8_t *valid) {
  if (!space_ok(sp) || !pipeline_ok(stages, S) || stage < 0 || stage >= S) return OVF_EINVAL;
  int64_t M = ovf_dense_count(sp);
  int n = stage > 0 ? stage : 1;
  ovf_state *st = (ovf_state *)calloc((size_t)n, sizeof(ovf_state));
  int32_t *cf = (int32_t *)calloc((size_t)n * 64, sizeof(int32_t));
  if (!st || !cf) { free(st); free(cf); return OVF_ENOMEM; }
  int rc = replay(stages, S, sp, prefix_cids, stage, st, cf);
  if (rc == OVF_OK) {
    decision d = { stages, S, sp, stage, st, cf };
#pragma omp parallel for schedule(static)
    for (int64_t cid = 0; cid < M; ++cid) {
      int32_t core[64];
      valid[cid] = (uint8_t)candidate(&d, cid, NULL, core, NULL);
      sequence_of(&d, core, x + (size_t)cid * S * 64);
    }
  }
  free(st); free(cf);
  return rc;
}

/* V of every valid candidate state of decision d under the recurrent network: the
 * sequences of the valid candidates, one after the other, through ovf_score_lstm.
 * sc[cid] = +inf and ok[cid] = 0 for the others. */
static int score_decision_lstm(const decision *d, const ovf_model *m, const float *weights,
                               float *sc, uint8_t *ok) {
  const int64_t M = ovf_dense_count(d->sp);
  const int S = d->S;
  int64_t nv = 0;
  for (int64_t cid = 0; cid < M; ++cid) {
    int32_t core[64];
    ok[cid] = (uint8_t)candidate(d, cid, NULL, core, NULL);
    sc[cid] = INFINITY;
    nv += ok[cid];
  }
  if (nv == 0) return OVF_OK;
  uint16_t *x = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)nv * S * 64);
  float *v = (float *)malloc(sizeof(float) * (size_t)nv);
  if (!x || !v) { free(x); free(v); return OVF_ENOMEM; }
  int64_t k = 0;
  for (int64_t cid = 0; cid < M; ++cid) {
    if (!ok[cid]) continue;
    int32_t core[64];
    candidate(d, cid, NULL, core, NULL);
    sequence_of(d, core, x + (size_t)k * S * 64);
    ++k;
  }
  int rc = ovf_score_lstm(m, weights, x, nv, S, v);
  k = 0;
  if (rc == OVF_OK)
    for (int64_t cid = 0; cid < M; ++cid)
      if (ok[cid]) sc[cid] = v[k++];
  free(x); free(v);
  return rc;
}

/* ----------------------------------------------------------------- argmin */

/* Inner loop of Algorithm 1 over ids [0, M) (or per consecutive block of `group`
 * ids when group > 0): v starts at +infinity and a candidate wins only if its score
 * is strictly smaller, so the first minimum is kept and NaN never wins.  Entries
 * with valid[n] == 0 are skipped (valid may be NULL).  No winner: index -1, +inf.
 * Indices are global ids. */
int ovf_argmin(const float *scores, const uint8_t *valid, int64_t M, int32_t group,
               int32_t *best_idx, float *best_val) {
  if (M < 0 || group < 0) return OVF_EINVAL;
  int64_t g = group > 0 ? group : (M > 0 ? M : 1);
  int64_t ng = (M + g - 1) / g;
  if (M == 0 && group == 0) ng = 1;
  for (int64_t k = 0; k < ng; ++k) {
    float v = INFINITY;
    int32_t s = -1;
    int64_t hi = (k + 1) * g < M ? (k + 1) * g : M;
    for (int64_t n = k * g; n < hi; ++n) {
      if (valid && !valid[n]) continue;
      if (scores[n] < v) { v = scores[n]; s = (int32_t)n; }
    }
    best_idx[k] = s;
    best_val[k] = v;
  }
  return OVF_OK;
}

/* ------------------------------------------------------------------ noise */

/* Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random
 * numbers: as easy as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplications
 * and xors on a 128-bit counter, the 64-bit key bumped by the Weyl constants between
 * rounds. */
void ovf_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Noise in [-1, 1) attached to (rollout, layer, candidate): the first Philox word of
 * counter (cid, stage, rollout, 0) under key = seed, top 24 bits, as k * 2^-23 - 1. */
float ovf_noise(uint64_t seed, int32_t rollout, int32_t stage, int32_t cid) {
  uint32_t ctr[4] = { (uint32_t)cid, (uint32_t)stage, (uint32_t)rollout, 0u };
  uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) }, out[4];
  ovf_philox4x32_10(ctr, key, out);
  return (float)(out[0] >> 8) * 0x1p-23f - 1.0f;
}

/* ----------------------------------------------------------------- greedy */

/* V(s) of every candidate state of one decision (the inner loop of Algorithm 1 before the
 * scan): sc[cid] for cid < M, ok[cid] = validity; the score of an invalid id is left
 * unspecified (the callback path sets +inf).  xcol is scratch of F * M values.  With
 * eps != 0 the exploration noise of Section 3.1 for (rollout, layer, candidate) is added
 * to the valid ones: one float multiply, one float add. */
static int decision_scores(const decision *dp, const ovf_model *m, const float *weights, ovf_vfun vfun,
                           void *user, int recurrent, float eps, uint64_t seed, int32_t rollout,
                           int32_t *xcol, float *sc, uint8_t *ok) {
  const decision d = *dp;
  const ovf_stage *stages = d.stages;
  const ovf_space *sp = d.sp;
  const int S = d.S, i = d.i, F = sp->F;
  const int32_t *cf = d.cf;
  const int64_t M = ovf_dense_count(sp);
  int rc = OVF_OK;
  {
    int32_t nb[192];
    memset(nb, 0, sizeof nb);
    for (int k = 1; k <= 3; ++k) {
      if (i - k >= 0)
        for (int t = 0; t < 48; ++t) nb[48 * (k - 1) + t] = cf[64 * (size_t)(i - k) + t];
      if (i + k < S) intrinsic(stages, S, i + k, nb + 144 + 16 * (k - 1));
    }
    /* features of every candidate state, column-per-candidate for the scorer */
    if (!recurrent) {
#pragma omp parallel for schedule(static)
      for (int64_t cid = 0; cid < M; ++cid) {
        int32_t core[64];
        ok[cid] = (uint8_t)candidate(&d, cid, NULL, core, NULL);
        for (int k = 0; k < 64; ++k) xcol[(size_t)k * M + cid] = core[k];
        if (F == 256)
          for (int k = 0; k < 192; ++k) xcol[(size_t)(64 + k) * M + cid] = nb[k];
      }
    }
    if (recurrent) {
      rc = score_decision_lstm(&d, m, weights, sc, ok);
      if (rc != OVF_OK) return rc;
    } else if (vfun) {
      for (int64_t cid = 0; cid < M; ++cid) {
        if (!ok[cid]) { sc[cid] = INFINITY; continue; }
        int32_t core[64];
        for (int k = 0; k < 64; ++k) core[k] = xcol[(size_t)k * M + cid];
        sc[cid] = (float)vfun(user, i, (int32_t)cid, core);
      }
    } else {
      rc = ovf_score_mlp(m, weights, xcol, M, M, sc);
      if (rc != OVF_OK) return rc;
    }
    /* Section 3.1: exploration adds a small random noise to the predictions */
    if (eps != 0.0f)
      for (int64_t cid = 0; cid < M; ++cid)
        if (ok[cid]) {
          float t = eps * ovf_noise(seed, rollout, i, (int32_t)cid);
          sc[cid] = sc[cid] + t;
        }
  }
  return rc;
}


/* Algorithm 1 over stages first..last with stages 0..first-1 already committed to
 * cids[0..first-1].  V is the MLP `m` (raw features -> normalise -> network), the
 * recurrent network `m` over the state's sequence form (model kind 1 with 64 inputs per
 * timestep), or the callback `vfun` when it is not NULL.  forced[i] >= 0 (forced may be NULL) replaces
 * the argmin of stage i by that candidate (used to follow a GPU decision that lies
 * inside the tolerance margin); top2[i] receives the second smallest score.
 * On return cids/values/states hold s_1..s_n; a stage with no winner gets -1 / +inf
 * and ends the schedule.  n_evals counts V evaluations (Section 2: N*M, not M^N). */
static int greedy_impl(const ovf_stage *stages, int S, const ovf_space *sp, const ovf_model *m,
                       const float *weights, ovf_vfun vfun, void *user, int first, int last,
                       const int32_t *forced, int32_t *cids, float *values, float *top2,
                       ovf_state *states, int64_t *n_evals, float eps, uint64_t seed, int32_t rollout) {
  if (!space_ok(sp) || !pipeline_ok(stages, S)) return OVF_EINVAL;
  if (first < 0 || last >= S || first > last + 1) return OVF_EINVAL;
  const int recurrent = !vfun && lstm_ok(m) && m->dims[0] == 64;
  if (!vfun && !recurrent && (!mlp_ok(m) || m->dims[0] != sp->F)) return OVF_EINVAL;
  const int64_t M = ovf_dense_count(sp);
  const int F = sp->F;
  ovf_state *st = (ovf_state *)calloc((size_t)S, sizeof(ovf_state));
  int32_t *cf = (int32_t *)calloc((size_t)S * 64, sizeof(int32_t));
  float *sc = (float *)malloc(sizeof(float) * (size_t)M);
  uint8_t *ok = (uint8_t *)malloc((size_t)M);
  int32_t *xcol = (int32_t *)malloc(sizeof(int32_t) * (size_t)F * (size_t)M);
  if (!st || !cf || !sc || !ok || !xcol) {
    free(st); free(cf); free(sc); free(ok); free(xcol);
    return OVF_ENOMEM;
  }
  int64_t evals = 0;
  int rc = replay(stages, S, sp, cids, first, st, cf);
  int dead = 0;
  for (int i = first; rc == OVF_OK && i <= last; ++i) {
    if (dead) {
      cids[i] = -1; values[i] = INFINITY;
      if (top2) top2[i] = INFINITY;
      continue;
    }
    decision d = { stages, S, sp, i, st, cf };
    rc = decision_scores(&d, m, weights, vfun, user, recurrent, eps, seed, rollout, xcol, sc, ok);
    if (rc != OVF_OK) break;
    /* the scan of Algorithm 1 */
    float v = INFINITY, v2 = INFINITY;
    int32_t s = -1;
    for (int64_t cid = 0; cid < M; ++cid) {
      if (!ok[cid]) continue;
      ++evals;
      if (sc[cid] < v) { v2 = v; v = sc[cid]; s = (int32_t)cid; }
      else if (sc[cid] < v2) v2 = sc[cid];
    }
    if (forced && forced[i] >= 0 && forced[i] < M && ok[forced[i]]) {
      s = forced[i];
      v = sc[s];
    }
    cids[i] = s; values[i] = v;
    if (top2) top2[i] = v2;
    if (s < 0) { dead = 1; continue; }
    candidate(&d, s, NULL, cf + 64 * (size_t)i, &st[i]);
  }
  if (rc == OVF_OK) {
    if (states) memcpy(states, st, sizeof(ovf_state) * (size_t)S);
    if (n_evals) *n_evals = evals;
  }
  free(st); free(cf); free(sc); free(ok); free(xcol);
  return rc;
}

int ovf_greedy(const ovf_stage *stages, int S, const ovf_space *sp, const ovf_model *m,
               const float *weights, ovf_vfun vfun, void *user, int first, int last,
               const int32_t *forced, int32_t *cids, float *values, float *top2,
               ovf_state *states, int64_t *n_evals) {
  return greedy_impl(stages, S, sp, m, weights, vfun, user, first, last, forced, cids, values, top2,
                     states, n_evals, 0.0f, 0, 0);
}

/* BestSchedule(n, V_eps) of Algorithm 2 / Section 3.1: the greedy scan with a small
 * random noise added to every prediction, n_rollouts times.  Rollout k adds
 * eps * ovf_noise(seed, first_rollout + k, layer, candidate) to the score (one float
 * multiply, one float add) before the scan; the kept value is the noisy one.
 * cids / values / top2 are [n_rollouts][S]; forced (nullable, [n_rollouts][S]) as in
 * ovf_greedy. */
int ovf_rollouts(const ovf_stage *stages, int S, const ovf_space *sp, const ovf_model *m,
                 const float *weights, float eps, uint64_t seed, int32_t first_rollout,
                 int32_t n_rollouts, const int32_t *forced, int32_t *cids, float *values, float *top2) {
  if (n_rollouts < 0) return OVF_EINVAL;
  for (int32_t k = 0; k < n_rollouts; ++k) {
    int rc = greedy_impl(stages, S, sp, m, weights, NULL, NULL, 0, S - 1,
                         forced ? forced + (size_t)k * S : NULL, cids + (size_t)k * S,
                         values + (size_t)k * S, top2 ? top2 + (size_t)k * S : NULL, NULL, NULL, eps, seed,
                         first_rollout + k);
    if (rc != OVF_OK) return rc;
  }
  return OVF_OK;
}

/* The scores the scan of decision `stage` sees, given the committed prefix
 * prefix_cids[0..stage-1]: scores[cid] (with the noise of (rollout, stage, cid) when
 * eps != 0) and valid[cid] for every cid < M.  Same arithmetic as ovf_greedy /
 * ovf_rollouts (it is the routine they call); lets a test look at the margin between any
 * two candidates of a decision, not only at the two smallest. */
int ovf_decision_scores(const ovf_stage *stages, int S, const ovf_space *sp, const ovf_model *m,
                        const float *weights, const int32_t *prefix_cids, int stage, float eps,
                        uint64_t seed, int32_t rollout, float *scores, uint8_t *valid) {
  if (!space_ok(sp) || !pipeline_ok(stages, S)) return OVF_EINVAL;
  if (stage < 0 || stage >= S) return OVF_EINVAL;
  const int recurrent = lstm_ok(m) && m->dims[0] == 64;
  if (!recurrent && (!mlp_ok(m) || m->dims[0] != sp->F)) return OVF_EINVAL;
  const int64_t M = ovf_dense_count(sp);
  ovf_state *st = (ovf_state *)calloc((size_t)S, sizeof(ovf_state));
  int32_t *cf = (int32_t *)calloc((size_t)S * 64, sizeof(int32_t));
  int32_t *xcol = (int32_t *)malloc(sizeof(int32_t) * (size_t)sp->F * (size_t)M);
  int rc = (st && cf && xcol) ? replay(stages, S, sp, prefix_cids, stage, st, cf) : OVF_ENOMEM;
  if (rc == OVF_OK) {
    decision d = { stages, S, sp, stage, st, cf };
    rc = decision_scores(&d, m, weights, NULL, NULL, recurrent, eps, seed, rollout, xcol, scores, valid);
  }
  free(st); free(cf); free(xcol);
  return rc;
}

/* ------------------------------------------------------------ beam search */

typedef struct { float v; int32_t beam; int32_t cid; } beam_item;

static int beam_item_less(const void *pa, const void *pb) {
  const beam_item *a = (const beam_item *)pa, *b = (const beam_item *)pb;
  if (a->v < b->v) return -1;
  if (a->v > b->v) return 1;
  if (a->beam != b->beam) return a->beam < b->beam ? -1 : 1;
  if (a->cid != b->cid) return a->cid < b->cid ? -1 : 1;
  return 0;
}

/* Beam search guided by V (the other search that Sections 3.1 and 4.1 run with the value
 * function, next to the greedy scan): keep the `width` best partial schedules per layer instead of one.
 * Layer by layer, every kept partial schedule is extended by every valid candidate of
 * the next layer, each extension is scored by V, and the `width` smallest scores
 * survive (ties: lower parent index, then lower candidate id; +inf and NaN never
 * survive).  width = 1 is Algorithm 1.  cids / values are [width][S] (value of the
 * state after each layer); rows are ordered by the score of the last layer reached;
 * unused rows and layers are -1 / +inf.  *n_beams = surviving schedules at the end. */
int ovf_beam(const ovf_stage *stages, int S, const ovf_space *sp, const ovf_model *m,
             const float *weights, ovf_vfun vfun, void *user, int width, int32_t *cids,
             float *values, int32_t *n_beams, int64_t *n_evals) {
  if (!space_ok(sp) || !pipeline_ok(stages, S) || width < 1) return OVF_EINVAL;
  const int recurrent = !vfun && lstm_ok(m) && m->dims[0] == 64;
  if (!vfun && !recurrent && (!mlp_ok(m) || m->dims[0] != sp->F)) return OVF_EINVAL;
  const int64_t M = ovf_dense_count(sp), Mp = ovf_padded_count(sp);
  const int F = sp->F;
  int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * (size_t)width * S);
  float *curv = (float *)malloc(sizeof(float) * (size_t)width * S);
  int32_t *nxt = (int32_t *)malloc(sizeof(int32_t) * (size_t)width * S);
  float *nxtv = (float *)malloc(sizeof(float) * (size_t)width * S);
  beam_item *items = (beam_item *)malloc(sizeof(beam_item) * (size_t)width * (size_t)M);
  int32_t *feat = (int32_t *)malloc(sizeof(int32_t) * (size_t)F * (size_t)Mp);
  float *sc = (float *)malloc(sizeof(float) * (size_t)M);
  if (!cur || !curv || !nxt || !nxtv || !items || !feat || !sc) {
    free(cur); free(curv); free(nxt); free(nxtv); free(items); free(feat); free(sc);
    return OVF_ENOMEM;
  }
  for (size_t k = 0; k < (size_t)width * S; ++k) { cur[k] = -1; curv[k] = INFINITY; }
  int live = 1; /* the empty schedule s_0 */
  int64_t evals = 0;
  int rc = OVF_OK;
  for (int i = 0; i < S && live > 0 && rc == OVF_OK; ++i) {
    size_t n_items = 0;
    for (int b = 0; b < live && rc == OVF_OK; ++b) {
      rc = ovf_featurize(stages, S, sp, cur + (size_t)b * S, i, feat);
      if (rc != OVF_OK) break;
      if (vfun) {
        for (int64_t cid = 0; cid < M; ++cid) {
          int32_t core[64];
          for (int k = 0; k < 64; ++k) core[k] = feat[(size_t)k * Mp + cid];
          sc[cid] = core[16] ? (float)vfun(user, i, (int32_t)cid, core) : INFINITY;
        }
      } else if (recurrent) {
        ovf_state *bst = (ovf_state *)calloc((size_t)(i > 0 ? i : 1), sizeof(ovf_state));
        int32_t *bcf = (int32_t *)calloc((size_t)(i > 0 ? i : 1) * 64, sizeof(int32_t));
        uint8_t *bok = (uint8_t *)malloc((size_t)M);
        if (!bst || !bcf || !bok) rc = OVF_ENOMEM;
        if (rc == OVF_OK) rc = replay(stages, S, sp, cur + (size_t)b * S, i, bst, bcf);
        if (rc == OVF_OK) {
          decision d = { stages, S, sp, i, bst, bcf };
          rc = score_decision_lstm(&d, m, weights, sc, bok);
        }
        free(bst); free(bcf); free(bok);
        if (rc != OVF_OK) break;
      } else {
        rc = ovf_score_mlp(m, weights, feat, Mp, M, sc);
        if (rc != OVF_OK) break;
      }
      for (int64_t cid = 0; cid < M; ++cid) {
        if (!feat[(size_t)16 * Mp + cid]) continue;
        ++evals;
        if (sc[cid] < INFINITY) { /* false for NaN too */
          items[n_items].v = sc[cid]; items[n_items].beam = b; items[n_items].cid = (int32_t)cid;
          ++n_items;
        }
      }
    }
    if (rc != OVF_OK) break;
    qsort(items, n_items, sizeof(beam_item), beam_item_less);
    int keep = n_items < (size_t)width ? (int)n_items : width;
    for (size_t k = 0; k < (size_t)width * S; ++k) { nxt[k] = -1; nxtv[k] = INFINITY; }
    for (int j = 0; j < keep; ++j) {
      const beam_item *it = &items[j];
      memcpy(nxt + (size_t)j * S, cur + (size_t)it->beam * S, sizeof(int32_t) * (size_t)i);
      memcpy(nxtv + (size_t)j * S, curv + (size_t)it->beam * S, sizeof(float) * (size_t)i);
      nxt[(size_t)j * S + i] = it->cid;
      nxtv[(size_t)j * S + i] = it->v;
    }
    if (keep == 0) {
      /* nothing survives: the schedules found so far end here, in their order */
      break;
    }
    int32_t *t1 = cur; cur = nxt; nxt = t1;
    float *t2 = curv; curv = nxtv; nxtv = t2;
    live = keep;
  }
  if (rc == OVF_OK) {
    memcpy(cids, cur, sizeof(int32_t) * (size_t)width * S);
    memcpy(values, curv, sizeof(float) * (size_t)width * S);
    if (n_beams) *n_beams = live;
    if (n_evals) *n_evals = evals;
  }
  free(cur); free(curv); free(nxt); free(nxtv); free(items); free(feat); free(sc);
  return rc;
}

int ovf_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}

/* Caps the threads of the loops over candidates (timing a single thread next to all
 * cores); n < 1 is ignored.  Changes no result. */
void ovf_set_num_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}
