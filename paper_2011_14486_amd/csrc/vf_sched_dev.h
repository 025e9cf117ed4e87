// Device-side candidate model shared by the featurize kernels and the fused scorer:
// saturating integer helpers, the per-decision context (what all candidates of one
// decision have in common) and the evaluation of one candidate state (Table 1 digits,
// validity under the committed loop structure of Sec. 2, the 64 core features of
// Sec. 3.2).  Include inside an anonymous namespace of a HIP translation unit.
#pragma once

constexpr uint32_t SATMAX = 2147483647u;

__device__ __forceinline__ uint32_t smul(uint32_t a, uint32_t b) {
  uint64_t p = (uint64_t)a * (uint64_t)b;
  return p > (uint64_t)SATMAX ? SATMAX : (uint32_t)p;
}
__device__ __forceinline__ uint32_t sadd(uint32_t a, uint32_t b) {
  uint32_t s = a + b;  // both <= 2^31-1: no wrap
  return s > SATMAX ? SATMAX : s;
}
__device__ __forceinline__ uint32_t cdiv(uint32_t a, uint32_t b) { return (a + b - 1u) / b; }
// 16 * num / den in fixed point; the numerator saturates before the division
__device__ __forceinline__ uint32_t ratio16(uint32_t num, uint32_t den) {
  uint32_t n16 = num > (SATMAX >> 4) ? SATMAX : (num << 4);
  return n16 / (den ? den : 1u);
}
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// r / n for a divisor n >= 1 with rcp = 1.0f / n, a handful of instructions instead of an
// integer division: below 2^24 the dividend is a float, the product is less than one away
// from the quotient, and one compare either way puts it right.
__device__ __forceinline__ uint32_t div_small(uint32_t r, uint32_t n, float rcp) {
  if (r >= (1u << 24)) return r / n;
  uint32_t q = (uint32_t)((float)r * rcp);
  if (q * n > r) --q;
  else if ((q + 1u) * n <= r) ++q;
  return q;
}

struct Tables {
  const int32_t *space, *stages, *intr, *suffix;
  int32_t *states, *cf, *prefix, *cids, *alive, *err;
  float *vals;
  int S;
};

// What is common to every candidate of one decision (one problem, one stage).
struct Dec {
  int32_t srec[16];
  int32_t intr[16];
  uint32_t E[3][3];   // region per instance when computed at ROOT, L1, L2
  uint32_t inst[3];   // number of instances at ROOT, L1, L2
  uint32_t inl_inst;  // number of evaluations when inlined into the anchor
  int32_t lvl_ok[4];  // compute_at level offered by the committed loop structure
  int32_t a_tp, a_nt, a_cat, a_perm, anchored;
  int32_t pm, pb, sm, spt;
  int32_t nb[192];    // rows 64..255 of the 256-feature layout
};

// Intrinsic block of one stage record (schedule-invariant, Sec. 3.2).
[[maybe_unused]] __device__ void intrinsic_of(const int32_t *w, int j, int S, int32_t *a) {
  uint32_t kind = w[0], W = w[1], H = w[2], C = w[3], RC = w[4], KH = w[5], KW = w[6];
  uint32_t stride = w[7], eb = w[12];
  uint32_t R = smul(smul(RC, KH), KW);
  uint32_t points = smul(smul(W, H), C);
  bool conv_like = (kind == VF_CONV || kind == VF_DWCONV);
  uint32_t macs = conv_like ? smul(points, R) : points;
  uint32_t cin = (kind == VF_CONV) ? RC : C;
  uint32_t in_elems = smul(smul(smul(W, stride), smul(H, stride)), cin);
  if (kind == VF_ADD) in_elems = smul(in_elems, 2u);
  uint32_t w_elems = 0;
  if (kind == VF_CONV) w_elems = smul(smul(smul(C, RC), KH), KW);
  else if (kind == VF_DWCONV) w_elems = smul(smul(C, KH), KW);
  a[0] = kind; a[1] = W; a[2] = H; a[3] = C;
  a[4] = R; a[5] = smul(KH, KW); a[6] = stride;
  a[7] = points; a[8] = macs; a[9] = in_elems; a[10] = w_elems;
  a[11] = smul(points, eb);
  a[12] = ratio16(macs, sadd(sadd(in_elems, w_elems), points));
  a[13] = w[9]; a[14] = j; a[15] = S - 1 - j;
}

// Region of the producer needed by a consumer box, clipped to the producer's extents.
__device__ void needed(const int32_t *srec, const int32_t *arec, const uint32_t box[3], uint32_t E[3]) {
  uint32_t sa = arec[7], kh = arec[5], kw = arec[6];
  E[0] = umin((uint32_t)srec[1], sadd(smul(box[0] - 1u, sa), kw));
  E[1] = umin((uint32_t)srec[2], sadd(smul(box[1] - 1u, sa), kh));
  E[2] = (arec[0] == VF_CONV) ? (uint32_t)srec[3] : umin((uint32_t)srec[3], box[2]);
}

// What the decision for one stage has just produced, for a caller that builds the next
// stage's context before those rows are in memory (they are in LDS): the stage's 64 committed
// features, its state record, the running sums behind it, and whether the problem goes on.
// stage < 0: nothing is overridden.
struct FreshRows {
  int stage;
  const int32_t *cf;   // [64]
  const int32_t *st;   // [16]
  int32_t pm, pb, alive;
};

// One thread: what the decision context derives from the rows it was given - the regions and
// instance counts per compute_at level from the anchor's committed loop structure, the levels
// on offer, the anchor's context features, the running sums.  ast / arec: the anchor's state
// record and stage record (read only if the stage has an anchor before it); acf: its committed
// features, all 64 or (packed) just entries 42, 54, 32, 23.
__device__ __forceinline__ void dec_derive(Dec &d, const vf_space &sp, int stage, int alive, const int32_t *ast,
                                           const int32_t *arec, const int32_t *acf, bool packed, int32_t pm, int32_t pb,
                                           int32_t sm, int32_t spt) {
  const int a = d.srec[8], kind = d.srec[0];
  d.E[0][0] = d.srec[1]; d.E[0][1] = d.srec[2]; d.E[0][2] = d.srec[3];
  d.inst[0] = 1;
  for (int l = 1; l < 3; ++l) {
    d.E[l][0] = d.E[0][0]; d.E[l][1] = d.E[0][1]; d.E[l][2] = d.E[0][2];
    d.inst[l] = 1;
  }
  d.inl_inst = 1;
  d.lvl_ok[0] = alive; d.lvl_ok[1] = 0; d.lvl_ok[2] = 0; d.lvl_ok[3] = 0;
  d.a_tp = d.a_nt = d.a_cat = d.a_perm = 0;
  bool anchored = (a >= 0 && a < stage && ast[15] == 1);
  d.anchored = anchored;
  if (anchored) {
    uint32_t fa[3] = {(uint32_t)ast[0], (uint32_t)ast[1], (uint32_t)ast[2]};
    uint32_t Ea[3] = {(uint32_t)ast[8], (uint32_t)ast[9], (uint32_t)ast[10]};
    uint32_t Oa[3] = {(uint32_t)ast[12], (uint32_t)ast[13], (uint32_t)ast[14]};
    uint32_t inst_a = ast[11];
    int d0 = sp.perm[ast[3]][0];
    uint32_t box[3] = {Ea[0], Ea[1], Ea[2]};
    box[d0] = fa[d0];
    needed(d.srec, arec, box, d.E[1]);
    d.inst[1] = smul(inst_a, Oa[d0]);
    needed(d.srec, arec, fa, d.E[2]);
    uint32_t tiles_a = smul(smul(Oa[0], Oa[1]), Oa[2]);
    d.inst[2] = smul(inst_a, tiles_a);
    uint32_t pp = 1;
    for (int k = 0; k < 3; ++k) pp = smul(smul(pp, Oa[k]), fa[k]);
    uint32_t Ra = smul(smul((uint32_t)arec[4], (uint32_t)arec[5]), (uint32_t)arec[6]);
    d.inl_inst = smul(smul(inst_a, pp), Ra);
    bool single = (d.srec[9] == 1) && alive;
    bool loops = (ast[6] != VF_INLINE);
    d.lvl_ok[1] = single && loops && Oa[d0] > 1u;
    d.lvl_ok[2] = single && loops && tiles_a > 1u;
    d.lvl_ok[3] = single && (kind == VF_POINTWISE || kind == VF_ADD);
    d.a_tp = acf[packed ? 0 : 42]; d.a_nt = acf[packed ? 1 : 54]; d.a_cat = acf[packed ? 2 : 32]; d.a_perm = acf[packed ? 3 : 23];
  }
  d.pm = pm;
  d.pb = pb;
  d.sm = sm;
  d.spt = spt;
}

// Cooperative set-up of the decision context for problem b, stage `stage`, in three steps with
// a workgroup barrier between them: every word that comes from memory is fetched by a thread of
// its own, in two rounds (the anchor's rows need the stage record first), and one thread then
// works on LDS only.  Rows of stage `fresh` are left out of the fetches: dec_finish takes them
// from fr (a caller that has just decided that stage can run the two fetch rounds before it
// knows the winner).
struct DecScratch {
  int32_t sc[8];  // alive, prefix sums (2), suffix sums (2)
  int32_t ast[16], arec[16], acf[4];
};

__device__ void dec_fetch_rows(Dec &d, vf_space &sp, DecScratch &ds, const Tables &t, int b, int stage, int fresh) {
  const int tid = threadIdx.x, nt = blockDim.x, S = t.S;
  const size_t row = (size_t)b * S;
  for (int i = tid; i < (int)(sizeof(vf_space) / 4); i += nt) ((int32_t *)&sp)[i] = t.space[i];
  if (tid < 16) {
    d.srec[tid] = t.stages[(row + stage) * 16 + tid];
    d.intr[tid] = t.intr[(row + stage) * 16 + tid];
  }
  for (int i = tid; i < 192; i += nt) {
    int32_t v = 0;
    if (i < 144) {
      int k = i / 48 + 1, f = i % 48;
      if (stage - k >= 0 && stage - k != fresh) v = t.cf[(row + stage - k) * 64 + f];
    } else {
      int k = (i - 144) / 16 + 1, f = (i - 144) % 16;
      if (stage + k < S) v = t.intr[(row + stage + k) * 16 + f];
    }
    d.nb[i] = v;
  }
  // (the last five threads of the first wave: the first ones have the most to fetch above)
  if (tid == 59) ds.sc[0] = fresh >= 0 ? 0 : t.alive[b];
  if (tid == 60 || tid == 61) ds.sc[tid - 59] = fresh >= 0 ? 0 : t.prefix[((size_t)b * (S + 1) + stage) * 2 + (tid - 60)];
  if (tid == 62 || tid == 63) ds.sc[tid - 59] = t.suffix[(row + stage) * 2 + (tid - 62)];
}

__device__ void dec_fetch_anchor(const Dec &d, DecScratch &ds, const Tables &t, int b, int stage, int fresh) {
  const int tid = threadIdx.x, S = t.S;
  const size_t row = (size_t)b * S;
  const int a = d.srec[8];
  const bool fetch = a >= 0 && a < stage && a != fresh;
  if (tid < 16) ds.ast[tid] = fetch ? t.states[(row + a) * 16 + tid] : 0;
  else if (tid < 32) ds.arec[tid - 16] = (a >= 0 && a < stage) ? t.stages[(row + a) * 16 + tid - 16] : 0;
  else if (tid < 36) {
    const int f = tid == 32 ? 42 : tid == 33 ? 54 : tid == 34 ? 32 : 23;
    ds.acf[tid - 32] = fetch ? t.cf[(row + a) * 64 + f] : 0;
  }
}

__device__ void dec_finish(Dec &d, const vf_space &sp, DecScratch &ds, int stage, const FreshRows &fr) {
  const int tid = threadIdx.x, nt = blockDim.x;
  if (fr.stage >= 0) {
    // the rows of the stage decided last, from the caller
    const int k = stage - fr.stage;
    if (k >= 1 && k <= 3)
      for (int f = tid; f < 48; f += nt) d.nb[(k - 1) * 48 + f] = fr.cf[f];
    if (d.srec[8] == fr.stage) {
      if (tid < 16) ds.ast[tid] = fr.st[tid];
      else if (tid >= 32 && tid < 36) ds.acf[tid - 32] = fr.cf[tid == 32 ? 42 : tid == 33 ? 54 : tid == 34 ? 32 : 23];
    }
    if (tid == 59) { ds.sc[0] = fr.alive; ds.sc[1] = fr.pm; ds.sc[2] = fr.pb; }
    __syncthreads();
  }
  if (tid == 0) dec_derive(d, sp, stage, ds.sc[0], ds.ast, ds.arec, ds.acf, true, ds.sc[1], ds.sc[2], ds.sc[3], ds.sc[4]);
  __syncthreads();
}

__device__ void build_dec_from(Dec &d, vf_space &sp, const Tables &t, int b, int stage, const FreshRows &fr) {
  __shared__ DecScratch ds;
  dec_fetch_rows(d, sp, ds, t, b, stage, fr.stage);
  __syncthreads();
  dec_fetch_anchor(d, ds, t, b, stage, fr.stage);
  __syncthreads();
  dec_finish(d, sp, ds, stage, fr);
}

// The same context with one round of fetches and the rest read by the one thread that derives
// (a chain of three dependent fetches, but no per-thread addresses that a long kernel would
// have to keep or spill): the form the whole-schedule kernel uses.
__device__ void build_dec(Dec &d, vf_space &sp, const Tables &t, int b, int stage) {
  const int tid = threadIdx.x, nt = blockDim.x, S = t.S;
  const size_t row = (size_t)b * S;
  for (int i = tid; i < (int)(sizeof(vf_space) / 4); i += nt) ((int32_t *)&sp)[i] = t.space[i];
  if (tid < 16) {
    d.srec[tid] = t.stages[(row + stage) * 16 + tid];
    d.intr[tid] = t.intr[(row + stage) * 16 + tid];
  }
  for (int i = tid; i < 192; i += nt) {
    int32_t v = 0;
    if (i < 144) {
      int k = i / 48 + 1, f = i % 48;
      if (stage - k >= 0) v = t.cf[(row + stage - k) * 64 + f];
    } else {
      int k = (i - 144) / 16 + 1, f = (i - 144) % 16;
      if (stage + k < S) v = t.intr[(row + stage + k) * 16 + f];
    }
    d.nb[i] = v;
  }
  __syncthreads();
  if (tid == 0) {
    const int a = d.srec[8];
    const size_t arow = row + (a >= 0 && a < stage ? a : 0);
    dec_derive(d, sp, stage, t.alive[b], t.states + arow * 16, t.stages + arow * 16, t.cf + arow * 64, false,
               t.prefix[((size_t)b * (S + 1) + stage) * 2 + 0], t.prefix[((size_t)b * (S + 1) + stage) * 2 + 1],
               t.suffix[(row + stage) * 2 + 0], t.suffix[(row + stage) * 2 + 1]);
  }
  __syncthreads();
}

// Table 1 digits of a candidate id, least significant first.
struct Digits {
  uint32_t ix, iy, ic, ip, vec, par, icat, isat;
};
__device__ __forceinline__ Digits digits_of(const vf_space &sp, uint32_t cid) {
  Digits g;
  uint32_t r = cid;
  g.ix = r % (uint32_t)sp.nf[0]; r /= (uint32_t)sp.nf[0];
  g.iy = r % (uint32_t)sp.nf[1]; r /= (uint32_t)sp.nf[1];
  g.ic = r % (uint32_t)sp.nf[2]; r /= (uint32_t)sp.nf[2];
  g.ip = r % (uint32_t)sp.nperm; r /= (uint32_t)sp.nperm;
  g.vec = r % (uint32_t)sp.nvec; r /= (uint32_t)sp.nvec;
  g.par = r % (uint32_t)sp.npar; r /= (uint32_t)sp.npar;
  g.icat = r % (uint32_t)sp.ncat; r /= (uint32_t)sp.ncat;
  g.isat = r;
  return g;
}
// The same digits through div_small (for a single thread that has a chain of them to do).
__device__ __forceinline__ Digits digits_small(const vf_space &sp, uint32_t cid) {
  const uint32_t radix[7] = {(uint32_t)sp.nf[0], (uint32_t)sp.nf[1], (uint32_t)sp.nf[2], (uint32_t)sp.nperm,
                             (uint32_t)sp.nvec, (uint32_t)sp.npar, (uint32_t)sp.ncat};
  uint32_t dig[7], r = cid;
#pragma unroll
  for (int k = 0; k < 7; ++k) {
    const uint32_t q = div_small(r, radix[k], 1.0f / (float)radix[k]);
    dig[k] = r - q * radix[k];
    r = q;
  }
  Digits g;
  g.ix = dig[0]; g.iy = dig[1]; g.ic = dig[2]; g.ip = dig[3]; g.vec = dig[4]; g.par = dig[5]; g.icat = dig[6];
  g.isat = r;
  return g;
}
__device__ __forceinline__ uint32_t id_of(const vf_space &sp, const Digits &g) {
  uint32_t r = g.isat;
  r = r * (uint32_t)sp.ncat + g.icat;
  r = r * (uint32_t)sp.npar + g.par;
  r = r * (uint32_t)sp.nvec + g.vec;
  r = r * (uint32_t)sp.nperm + g.ip;
  r = r * (uint32_t)sp.nf[2] + g.ic;
  r = r * (uint32_t)sp.nf[1] + g.iy;
  return r * (uint32_t)sp.nf[0] + g.ix;
}
__device__ __forceinline__ uint32_t pack_digits(const Digits &g) {
  return g.ix | g.iy << 4 | g.ic << 8 | g.ip << 12 | g.vec << 16 | g.par << 20 | g.icat << 24 | g.isat << 28;
}
__device__ __forceinline__ Digits unpack_digits(uint32_t dec) {
  Digits g;
  g.ix = dec & 15u; g.iy = (dec >> 4) & 15u; g.ic = (dec >> 8) & 15u; g.ip = (dec >> 12) & 15u;
  g.vec = (dec >> 16) & 15u; g.par = (dec >> 20) & 15u; g.icat = (dec >> 24) & 15u; g.isat = dec >> 28;
  return g;
}

// The quotients of the evaluation that depend on a digit and the decision only, so that
// a kernel that evaluates many candidates of one decision can look them up: per level
// and dimension the tile count of every split factor and the parallel efficiency of that
// many tasks; per dimension the vector lanes and vector efficiency of every factor.
struct EvalTabs {
  uint32_t O[3][3][8];        // cdiv(E[level][dim], fac[dim][k])
  uint32_t par_eff[3][3][8];  // ratio16(O, cdiv(O, ncores) * ncores)
  uint32_t lanes[3][8];       // min(fac[dim][k], vlen)
  uint32_t vec_eff[3][8];     // ratio16(fac, cdiv(fac, vlen) * vlen)
  uint32_t par_eff1;          // the parallel efficiency of a single task
};
// first: the thread that takes entry 0 (the others follow it), for a caller whose first
// threads are busy with something else.
[[maybe_unused]] __device__ void fill_evaltabs(EvalTabs &tb, const Dec &d, const vf_space &sp, int first = 0) {
  for (int i = (int)threadIdx.x - first; i >= 0 && i < 72; i += blockDim.x) {
    const int lvl = i / 24, dd = (i / 8) % 3, k = i % 8;
    const uint32_t f = k < sp.nf[dd] ? (uint32_t)sp.fac[dd][k] : 1u;
    const uint32_t o = cdiv(d.E[lvl][dd], f);
    tb.O[lvl][dd][k] = o;
    tb.par_eff[lvl][dd][k] = ratio16(o, smul(cdiv(o, (uint32_t)sp.ncores), (uint32_t)sp.ncores));
    if (lvl == 0) {
      tb.lanes[dd][k] = umin(f, (uint32_t)sp.vlen);
      tb.vec_eff[dd][k] = ratio16(f, smul(cdiv(f, (uint32_t)sp.vlen), (uint32_t)sp.vlen));
    }
    if (i == 0) tb.par_eff1 = ratio16(1u, smul(cdiv(1u, (uint32_t)sp.ncores), (uint32_t)sp.ncores));
  }
}

// One candidate state from its digits: validity and (FEATS) the 64 core features.
// Rows 0..15 are always the stage's intrinsic block; rows 16..63 are zero when the
// candidate is not valid.  tb (nullable): the decision's quotient tables.
template <bool FEATS>
__device__ __forceinline__ bool eval_digits(const Dec &d, const vf_space &sp, const Digits &g, const EvalTabs *tb,
                                            int32_t *core) {
  const uint32_t ix = g.ix, iy = g.iy, ic = g.ic, ip = g.ip, vec = g.vec, par = g.par, isat = g.isat;
  const int cat = sp.cat[g.icat];
  const uint32_t hoist = isat;
  uint32_t f[3] = {(uint32_t)sp.fac[0][ix], (uint32_t)sp.fac[1][iy], (uint32_t)sp.fac[2][ic]};
  uint32_t E[3] = {1u, 1u, 1u};
  uint32_t inst;

  bool valid = d.lvl_ok[cat] != 0;
  if (cat == VF_INLINE) {
    valid = valid && ((ix | iy | ic | ip | vec | par | isat) == 0u);
    f[0] = f[1] = f[2] = 1u;
    inst = d.inl_inst;
  } else {
    E[0] = d.E[cat][0]; E[1] = d.E[cat][1]; E[2] = d.E[cat][2];
    inst = d.inst[cat];
    valid = valid && hoist <= (uint32_t)cat && f[0] <= E[0] && f[1] <= E[1] && f[2] <= E[2];
  }
  if (!FEATS) return valid;

#pragma unroll
  for (int k = 0; k < 16; ++k) core[k] = d.intr[k];
  if (!valid) {
#pragma unroll
    for (int k = 16; k < 64; ++k) core[k] = 0;
    return false;
  }

  const int p0 = sp.perm[ip][0], p2 = sp.perm[ip][2];
  const uint32_t kind = d.srec[0], RC = d.srec[4], KH = d.srec[5], KW = d.srec[6];
  const uint32_t stride = d.srec[7], eb = d.srec[12];
  const uint32_t R = d.intr[4], points = d.intr[7];
  const bool looked_up = tb != nullptr && cat != VF_INLINE;
  const uint32_t idx[3] = {ix, iy, ic};
  uint32_t O[3];
  if (looked_up) {
    O[0] = tb->O[cat][0][ix]; O[1] = tb->O[cat][1][iy]; O[2] = tb->O[cat][2][ic];
  } else {
    O[0] = cdiv(E[0], f[0]); O[1] = cdiv(E[1], f[1]); O[2] = cdiv(E[2], f[2]);
  }

  core[16] = 1;
  core[17] = f[0]; core[18] = f[1]; core[19] = f[2];
  core[20] = O[0]; core[21] = O[1]; core[22] = O[2];
  core[23] = ip; core[24] = p2; core[25] = p0;
  core[26] = vec;
  const uint32_t fin = p2 == 0 ? f[0] : (p2 == 1 ? f[1] : f[2]);
  if (looked_up) {
    core[27] = vec ? tb->lanes[p2][idx[p2]] : 1u;
    core[28] = vec ? tb->vec_eff[p2][idx[p2]] : 16u;
  } else {
    core[27] = vec ? umin(fin, (uint32_t)sp.vlen) : 1u;
    core[28] = vec ? ratio16(fin, smul(cdiv(fin, (uint32_t)sp.vlen), (uint32_t)sp.vlen)) : 16u;
  }
  core[29] = par;
  const uint32_t Oout = p0 == 0 ? O[0] : (p0 == 1 ? O[1] : O[2]);
  const uint32_t tasks = par ? Oout : 1u;
  core[30] = tasks;
  if (tb != nullptr && !par) core[31] = tb->par_eff1;
  else if (looked_up) core[31] = tb->par_eff[cat][p0][idx[p0]];
  else core[31] = ratio16(tasks, smul(cdiv(tasks, (uint32_t)sp.ncores), (uint32_t)sp.ncores));
  core[32] = cat; core[33] = hoist;
  core[34] = E[0]; core[35] = E[1]; core[36] = E[2];
  core[37] = inst;
  uint32_t padded = smul(smul(smul(smul(smul(O[0], f[0]), O[1]), f[1]), O[2]), f[2]);
  core[38] = padded;
  uint32_t total_points = smul(inst, padded);
  core[39] = total_points;
  core[40] = smul(total_points, R);
  core[41] = ratio16(total_points, points);
  uint32_t tile_points = smul(smul(f[0], f[1]), f[2]);
  core[42] = tile_points;
  uint32_t tin = smul(sadd(smul(f[0] - 1u, stride), KW), sadd(smul(f[1] - 1u, stride), KH));
  tin = smul(tin, kind == VF_CONV ? RC : f[2]);
  if (kind == VF_ADD) tin = smul(tin, 2u);
  core[43] = tin;
  uint32_t tw = 0;
  if (kind == VF_CONV) tw = smul(smul(smul(f[2], RC), KH), KW);
  else if (kind == VF_DWCONV) tw = smul(smul(f[2], KH), KW);
  core[44] = tw;
  uint32_t ws = sadd(sadd(tile_points, tin), tw);
  core[45] = ws;
  uint32_t ws_bytes = smul(ws, eb);
  core[46] = ws_bytes <= (uint32_t)sp.l1_bytes;
  core[47] = ws_bytes <= (uint32_t)sp.l2_bytes;
  if (cat == VF_INLINE) {
    core[48] = 0; core[49] = 0; core[50] = 0;
  } else {
    const int lvl = cat - (int)hoist;  // where the buffer lives
    core[48] = smul(smul(d.E[lvl][0], d.E[lvl][1]), d.E[lvl][2]);
    core[49] = d.inst[lvl];
    core[50] = smul(total_points, eb);
  }
  uint32_t ntiles = smul(smul(O[0], O[1]), O[2]);
  core[51] = smul(smul(inst, ntiles), smul(sadd(tin, tw), eb));
  core[52] = p2 == 0 ? f[0] : 1u;
  core[53] = ratio16(smul(tile_points, R), sadd(tin, tw));
  core[54] = ntiles;
  core[55] = (O[0] * f[0] == E[0]) && (O[1] * f[1] == E[1]) && (O[2] * f[2] == E[2]);
  core[56] = d.a_tp; core[57] = d.a_nt; core[58] = d.a_cat;
  core[59] = d.anchored ? (int32_t)((int32_t)ip == d.a_perm) : 0;
  core[60] = d.pm; core[61] = d.pb; core[62] = d.sm; core[63] = d.spt;
  return true;
}

// One candidate state from its id: digits (packed into dec), validity and (FEATS) the
// 64 core features.
template <bool FEATS>
__device__ __forceinline__ bool eval_candidate(const Dec &d, const vf_space &sp, uint32_t cid,
                                               uint32_t &dec, int32_t *core) {
  const Digits g = digits_of(sp, cid);
  dec = pack_digits(g);
  return eval_digits<FEATS>(d, sp, g, nullptr, core);
}


// True when no candidate id in [lo, hi) can be valid, judged from the two most
// significant digits alone (compute_at level, store_at hoist: Table 1).  A level that
// is closed for the stage, or a hoist above the level, rules out a whole run of
// consecutive ids; inlining leaves one id per run.  False means "some id may be valid".
__device__ __forceinline__ bool range_closed(const Dec &d, const vf_space &sp, uint32_t lo, uint32_t hi) {
  if (hi <= lo) return true;
  const uint32_t run = (uint32_t)sp.nf[0] * (uint32_t)sp.nf[1] * (uint32_t)sp.nf[2] * (uint32_t)sp.nperm *
                       (uint32_t)sp.nvec * (uint32_t)sp.npar;  // ids per (level, hoist) pair
  const uint32_t q0 = lo / run, q1 = (hi - 1u) / run;
  if (q1 - q0 > 8u) return false;
  for (uint32_t q = q0; q <= q1; ++q) {
    const uint32_t icat = q % (uint32_t)sp.ncat, isat = q / (uint32_t)sp.ncat;
    const int cat = sp.cat[icat];
    if (d.lvl_ok[cat] == 0) continue;
    if (cat == VF_INLINE) {
      const uint32_t id = q * run;  // every other digit zero
      if (isat == 0u && id >= lo && id < hi) return false;
    } else if (isat <= (uint32_t)cat) {
      return false;
    }
  }
  return true;
}


// ---- normalisation (Sec. 3.2: the network is fed normalised feature values)

// piecewise-linear log2 of a non-negative integer: exponent + (significand - 1)
__device__ __forceinline__ float plog2_dev(int32_t x) {
  if (x <= 0) return 0.0f;
  float xf = (float)x;  // round to nearest even
  uint32_t u = __float_as_uint(xf);
  int e = (int)(u >> 23) - 127;
  float frac = __uint_as_float((u & 0x007fffffu) | 0x3f800000u) - 1.0f;  // exact
  return (float)e + frac;
}

typedef __bf16 vf_bf16x2 __attribute__((ext_vector_type(2)));
typedef float vf_floatx2 __attribute__((ext_vector_type(2)));

// two floats -> packed bfloat16 pair (round to nearest even, v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  vf_floatx2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, vf_bf16x2));
}

// ---- exploration noise (Sec. 3.1: a small random noise is added to the predictions)

// Philox4x32-10 (Salmon et al., SC'11), first output word
__device__ __forceinline__ uint32_t philox_first(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  return c0;
}

struct NoiseArgs {
  float eps;            // 0: no noise
  uint32_t k0, k1;      // seed
  int32_t stage;
  int32_t first_rollout;  // problem p is rollout first_rollout + p
};

// score + eps * u, u in [-1, 1) from the counter (candidate, layer, rollout)
__device__ __forceinline__ float add_noise(const NoiseArgs &na, float s, int p, int32_t cid) {
  const uint32_t x = philox_first((uint32_t)cid, (uint32_t)na.stage, (uint32_t)(na.first_rollout + p), 0u, na.k0, na.k1);
  const float u = (float)(x >> 8) * 0x1p-23f - 1.0f;
  return __fadd_rn(s, __fmul_rn(na.eps, u));
}

// The decision context in the form the fused scorer wants it: built once per problem
// and stage (by the commit of the stage before, or by k_prepare), fetched by every
// scoring workgroup with one coalesced copy.
//
// stat: the rows of the network's input that every candidate of the decision shares,
// normalised, as bf16 pairs, one group of 8 words per k-step of 16 rows of the first layer:
// words [0, 8) rows 0..15 (the stage's intrinsic block), [8, 16) rows 48..63 with the rows
// that do depend on the candidate (48..55, 59) left zero - i.e. the anchor's tile_points /
// n_tiles / compute_at level and the four running sums - and [16, 112) rows 64..255 (the
// neighbour stages).  Sec. 3.2 itself says that intrinsic features do not depend on the
// schedule: their part of the first layer is computed once per decision (fold_bias).
constexpr int VF_STAT_WORDS = 112;
struct DecPack {
  Dec d;
  vf_space sp;
  uint32_t stat[VF_STAT_WORDS];
  uint32_t pad[VF_DECPACK_DWORDS - (sizeof(Dec) + sizeof(vf_space)) / 4 - VF_STAT_WORDS];
};
static_assert(sizeof(DecPack) == VF_DECPACK_DWORDS * 4, "DecPack size");

// Word q of DecPack::stat from the decision context.
__device__ __forceinline__ uint32_t stat_word(const Dec &d, int q) {
  if (q >= 16) return pack_bf16(plog2_dev(d.nb[2 * (q - 16)]), plog2_dev(d.nb[2 * (q - 16) + 1]));
  if (q < 8) return pack_bf16(plog2_dev(d.intr[2 * q]), plog2_dev(d.intr[2 * q + 1]));
  // rows 48 + 2 (q - 8), 49 + 2 (q - 8): 56 a_tp, 57 a_nt, 58 a_cat, 59 the candidate's own, 60..63 the sums
  switch (q) {
    case 12: return pack_bf16(plog2_dev(d.a_tp), plog2_dev(d.a_nt));
    case 13: return pack_bf16(plog2_dev(d.a_cat), 0.0f);
    case 14: return pack_bf16(plog2_dev(d.pm), plog2_dev(d.pb));
    case 15: return pack_bf16(plog2_dev(d.sm), plog2_dev(d.spt));
    default: return 0u;
  }
}

// Builds the pack for (problem b, stage) in LDS (every thread of the block takes part).
[[maybe_unused]] __device__ void fill_decpack(DecPack &pk, const Tables &t, int b, int stage) {
  FreshRows none;
  none.stage = -1; none.cf = nullptr; none.st = nullptr; none.pm = none.pb = none.alive = 0;
  build_dec_from(pk.d, pk.sp, t, b, stage, none);  // (two rounds of fetches instead of three)
  for (int q = threadIdx.x; q < VF_STAT_WORDS; q += blockDim.x) pk.stat[q] = stat_word(pk.d, q);
  __syncthreads();
}

// Algorithm 1's "s_i := s": one thread records candidate c (value v) of problem b as
// the decision for `stage` - its derived loop structure, its 64 core features, the
// running sums - or, when there is no valid winner, ends that problem's schedule.
// d / sp are the decision context of (b, stage).
// tb (nullable): the decision's quotient tables, for a caller that has them at hand.
[[maybe_unused]] __device__ __forceinline__ void commit_winner(const Tables &t, const Dec &d, const vf_space &sp, int b, int stage,
                                               int32_t c, float v, uint32_t M, bool forced, const EvalTabs *tb = nullptr) {
  const int S = t.S;
  const size_t row = (size_t)b * S + stage;
  int32_t *pre = t.prefix + ((size_t)b * (S + 1) + stage) * 2;
  // (read before anything is stored: a load behind the stores would wait for all of them)
  const int32_t pre_m = pre[0], pre_b = pre[1];
  int32_t core[64];
  bool ok = false;
  if (c >= 0 && (uint32_t)c < M) {
    if (tb != nullptr) {
      ok = eval_digits<true>(d, sp, digits_small(sp, (uint32_t)c), tb, core);
    } else {
      uint32_t dec;
      ok = eval_candidate<true>(d, sp, (uint32_t)c, dec, core);
    }
  }
  if (!ok) {
    if (forced) t.err[0] = 1;
    t.alive[b] = 0;
    t.cids[row] = -1;
    t.vals[row] = __builtin_inff();
    pre[2] = pre_m; pre[3] = pre_b;
  } else {
#pragma unroll
    for (int k = 0; k < 64; ++k) t.cf[row * 64 + k] = core[k];
    int32_t *st = t.states + row * 16;
    st[0] = core[17]; st[1] = core[18]; st[2] = core[19];
    st[3] = core[23]; st[4] = core[26]; st[5] = core[29]; st[6] = core[32]; st[7] = core[33];
    st[8] = core[34]; st[9] = core[35]; st[10] = core[36];
    st[11] = core[37];
    st[12] = core[20]; st[13] = core[21]; st[14] = core[22];
    st[15] = 1;
    t.cids[row] = c;
    t.vals[row] = v;
    pre[2] = sadd((uint32_t)pre_m, (uint32_t)core[40]);
    pre[3] = sadd((uint32_t)pre_b, (uint32_t)core[50]);
  }
}

// commit_winner for a caller that goes on to the next decision by itself: the winner's rows are
// left in LDS (cf64, st16, and the values of a FreshRows record) for build_dec_from, and reach
// the tables only if `store` - every workgroup of a launch works them out, one of them writes.
// The running sums of the decision's own stage are taken from its context (d.pm, d.pb).
[[maybe_unused]] __device__ __forceinline__ void commit_winner_fresh(const Tables &t, const Dec &d, const vf_space &sp, int b,
                                                                   int stage, int32_t c, float v, uint32_t M,
                                                                   const EvalTabs &tb, bool store, int32_t *cf64,
                                                                   int32_t *st16, int32_t *sums3) {
  const int S = t.S;
  const size_t row = (size_t)b * S + stage;
  int32_t *pre = t.prefix + ((size_t)b * (S + 1) + stage) * 2;
  const int32_t pre_m = d.pm, pre_b = d.pb;
  int32_t core[64];
  bool ok = false;
  if (c >= 0 && (uint32_t)c < M) ok = eval_digits<true>(d, sp, digits_small(sp, (uint32_t)c), &tb, core);
  if (!ok) {
#pragma unroll
    for (int k = 0; k < 64; ++k) cf64[k] = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) st16[k] = 0;
    sums3[0] = pre_m; sums3[1] = pre_b; sums3[2] = 0;
    if (store) {
      t.alive[b] = 0;
      t.cids[row] = -1;
      t.vals[row] = __builtin_inff();
      pre[2] = pre_m; pre[3] = pre_b;
    }
  } else {
    int32_t st[16];
    st[0] = core[17]; st[1] = core[18]; st[2] = core[19];
    st[3] = core[23]; st[4] = core[26]; st[5] = core[29]; st[6] = core[32]; st[7] = core[33];
    st[8] = core[34]; st[9] = core[35]; st[10] = core[36];
    st[11] = core[37];
    st[12] = core[20]; st[13] = core[21]; st[14] = core[22];
    st[15] = 1;
    const int32_t pm = (int32_t)sadd((uint32_t)pre_m, (uint32_t)core[40]), pb = (int32_t)sadd((uint32_t)pre_b, (uint32_t)core[50]);
#pragma unroll
    for (int k = 0; k < 64; ++k) cf64[k] = core[k];
#pragma unroll
    for (int k = 0; k < 16; ++k) st16[k] = st[k];
    sums3[0] = pm; sums3[1] = pb; sums3[2] = d.lvl_ok[0];
    if (store) {
#pragma unroll
      for (int k = 0; k < 64; ++k) t.cf[row * 64 + k] = core[k];
#pragma unroll
      for (int k = 0; k < 16; ++k) t.states[row * 16 + k] = st[k];
      t.cids[row] = c;
      t.vals[row] = v;
      pre[2] = pm; pre[3] = pb;
    }
  }
}

// The same as a real call, for kernels whose main loop should not carry the registers of
// an inlined copy.  The table pointers that a commit touches come one by one, so that they
// travel in registers: a structure would go through the stack (scratch memory, a round trip
// to memory on either side of the call), a reference to it would be read again behind every
// store.
[[maybe_unused]] __device__ __attribute__((noinline)) void commit_winner_call(
    int32_t *states, int32_t *cf, int32_t *prefix, int32_t *cids, float *vals, int32_t *alive, int S, const Dec &d,
    const vf_space &sp, const EvalTabs &tb, int b, int stage, int32_t c, float v, uint32_t M) {
  Tables t;
  t.space = t.stages = t.intr = t.suffix = nullptr;
  t.states = states; t.cf = cf; t.prefix = prefix; t.cids = cids; t.alive = alive; t.err = nullptr;
  t.vals = vals;
  t.S = S;
  commit_winner(t, d, sp, b, stage, c, v, M, false, &tb);
}

// Builds the pack for (problem b, stage) in LDS and copies it to out[b].
[[maybe_unused]] __device__ void write_decpack(DecPack &pk, const Tables &t, int b, int stage, uint32_t *out) {
  fill_decpack(pk, t, b, stage);
  const uint32_t *src = reinterpret_cast<const uint32_t *>(&pk);
  const int used = (int)((sizeof(Dec) + sizeof(vf_space)) / 4 + VF_STAT_WORDS);
  for (int i = threadIdx.x; i < VF_DECPACK_DWORDS; i += blockDim.x)
    out[(size_t)b * VF_DECPACK_DWORDS + i] = i < used ? src[i] : 0u;
}

// Table pointers of a context.
inline Tables tables_of(const vf_ctx *c) {
  Tables t;
  t.space = c->d_space; t.stages = c->d_stages; t.intr = c->d_intr; t.suffix = c->d_suffix;
  t.states = c->d_states; t.cf = c->d_cf; t.prefix = c->d_prefix; t.cids = c->d_cids;
  t.alive = c->d_alive; t.err = c->d_err; t.vals = c->d_vals; t.S = c->S;
  return t;
}
