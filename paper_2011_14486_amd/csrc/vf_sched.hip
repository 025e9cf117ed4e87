// Candidate enumeration, featurization and commit kernels (gfx950).
//
// Algorithm 1 of the paper loops "for s in C_i" over the candidate states of layer
// L_i; here one GPU thread evaluates one candidate id.  A candidate is one choice for
// each primitive of Table 1; whether it is valid depends on the loop structure of
// the stages committed so far (Sec. 2), which is read from the per-problem state
// tables.  Everything that is the same for all candidates of a decision (the stage's
// intrinsic features, the region the stage must compute at each compute_at level of
// its anchor, the neighbour feature rows) is worked out once per workgroup and kept
// in LDS; the per-candidate part is integer arithmetic saturating at 2^31-1
// (Sec. 3.2: intrinsic and acquired features).
#include <utility>

#include "vf_internal.h"

namespace {

#include "vf_sched_dev.h"

// ------------------------------------------------------------------ kernels

__global__ __launch_bounds__(64) void k_setup(Tables t, int32_t *intr, int32_t *suffix) {
  const int b = blockIdx.x, S = t.S;
  const size_t row = (size_t)b * S;
  for (int j = threadIdx.x; j < S; j += blockDim.x) {
    int32_t a[16];
    intrinsic_of(t.stages + (row + j) * 16, j, S, a);
    for (int k = 0; k < 16; ++k) intr[(row + j) * 16 + k] = a[k];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t sm = 0, sp = 0;
    for (int j = S - 1; j >= 0; --j) {
      suffix[(row + j) * 2 + 0] = sm;
      suffix[(row + j) * 2 + 1] = sp;
      sm = sadd(sm, (uint32_t)intr[(row + j) * 16 + 8]);
      sp = sadd(sp, (uint32_t)intr[(row + j) * 16 + 7]);
    }
  }
}

__global__ __launch_bounds__(256) void k_reset(Tables t, int B) {
  const int S = t.S;
  const size_t n = (size_t)B * S;
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x, step = (size_t)gridDim.x * blockDim.x;
  for (size_t i = i0; i < n * 64; i += step) t.cf[i] = 0;
  for (size_t i = i0; i < n * 16; i += step) t.states[i] = 0;
  for (size_t i = i0; i < (size_t)B * (S + 1) * 2; i += step) t.prefix[i] = 0;
  for (size_t i = i0; i < n; i += step) { t.cids[i] = -1; t.vals[i] = __builtin_inff(); }
  for (size_t i = i0; i < (size_t)B; i += step) t.alive[i] = 1;
  if (i0 == 0) t.err[0] = 0;
}

// Back to the state in which stages 0..first-1 are committed and nothing behind them is:
// one workgroup per problem.
__global__ __launch_bounds__(256) void k_rewind(Tables t, int first) {
  const int S = t.S, b = blockIdx.x, tid = threadIdx.x;
  const size_t row = (size_t)b * S;
  for (int i = first * 64 + tid; i < S * 64; i += 256) t.cf[row * 64 + i] = 0;
  for (int i = first * 16 + tid; i < S * 16; i += 256) t.states[row * 16 + i] = 0;
  for (int i = (first + 1) * 2 + tid; i < (S + 1) * 2; i += 256) t.prefix[(size_t)b * (S + 1) * 2 + i] = 0;
  for (int i = first + tid; i < S; i += 256) { t.cids[row + i] = -1; t.vals[row + i] = __builtin_inff(); }
  if (tid == 0) t.alive[b] = first == 0 || t.cids[row + first - 1] >= 0;
}

__global__ __launch_bounds__(256) void k_fill_i32(int32_t *p, size_t n, int32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ __launch_bounds__(256) void k_enumerate(Tables t, int stage, uint32_t M, uint32_t Mpad,
                                                   uint32_t *dec_out, uint8_t *valid_out, int32_t *n_valid) {
  __shared__ Dec d;
  __shared__ vf_space sp;
  __shared__ int32_t wcount[4];
  const int b = blockIdx.y;
  build_dec(d, sp, t, b, stage);
  const uint32_t cid = blockIdx.x * 256u + threadIdx.x;
  uint32_t dec = 0;
  bool valid = false;
  if (cid < M) valid = eval_candidate<false>(d, sp, cid, dec, nullptr);
  if (dec_out) dec_out[(size_t)b * Mpad + cid] = dec;
  if (valid_out) valid_out[(size_t)b * Mpad + cid] = valid ? 1 : 0;
  if (n_valid) {
    unsigned long long m = __ballot(valid);
    if ((threadIdx.x & 63) == 0) wcount[threadIdx.x >> 6] = __popcll(m);
    __syncthreads();
    if (threadIdx.x == 0) {
      int c = wcount[0] + wcount[1] + wcount[2] + wcount[3];
      if (c) atomicAdd(&n_valid[b], c);  // integer sum: order does not matter
    }
  }
}

// Feature-major output feat[b][F][Mpad].  A workgroup covers SPAN consecutive blocks of 256
// candidates.  The 64 rows that differ from candidate to candidate go through LDS, 32 rows
// of a block at a time, so that every store instruction of a wave writes a kilobyte of one
// row (16 bytes per lane); the other rows are the same for every candidate and are written
// over the workgroup's whole span at once.
constexpr int VF_FEAT_SPAN = 4;
__global__ __launch_bounds__(256) void k_featurize(Tables t, int stage, uint32_t M, uint32_t Mpad, int F,
                                                   int32_t *feat) {
  __shared__ Dec d;
  __shared__ vf_space sp;
  __shared__ __attribute__((aligned(16))) int32_t tile[32][256];
  const int b = blockIdx.y;
  build_dec(d, sp, t, b, stage);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int32_t *out = feat + (size_t)b * F * Mpad;
  const uint32_t first = blockIdx.x * (uint32_t)(256 * VF_FEAT_SPAN);
  if (F == 256) {
    // rows 64..255: each wave writes its rows over the whole span (first: these stores need
    // no evaluation and are under way while the candidates are evaluated)
    for (int r = w; r < 192; r += 4) {
      const int32_t v = d.nb[r];
#pragma unroll
      for (int sb = 0; sb < VF_FEAT_SPAN; ++sb) {
        const uint32_t col0 = first + 256u * sb + 4u * lane;
        if (col0 >= Mpad) break;
        int4 q;
        q.x = col0 + 0 < M ? v : 0;
        q.y = col0 + 1 < M ? v : 0;
        q.z = col0 + 2 < M ? v : 0;
        q.w = col0 + 3 < M ? v : 0;
        *reinterpret_cast<int4 *>(out + (size_t)(64 + r) * Mpad + col0) = q;
      }
    }
  }
  for (int sb = 0; sb < VF_FEAT_SPAN; ++sb) {
    const uint32_t base = first + 256u * sb;
    if (base >= Mpad) break;
    const uint32_t cid = base + threadIdx.x;
    int32_t core[64];
    if (cid < M) {
      uint32_t dec;
      eval_candidate<true>(d, sp, cid, dec, core);
    } else {
#pragma unroll
      for (int k = 0; k < 64; ++k) core[k] = 0;
    }
    const uint32_t col0 = base + 4u * lane;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      __syncthreads();  // the tile has been read
#pragma unroll
      for (int k = 0; k < 32; ++k) tile[k][threadIdx.x] = core[32 * half + k];
      __syncthreads();
#pragma unroll
      for (int r = w; r < 32; r += 4)
        *reinterpret_cast<int4 *>(out + (size_t)(32 * half + r) * Mpad + col0) =
            *reinterpret_cast<const int4 *>(&tile[r][4 * lane]);
    }
  }
}

// One workgroup per problem: pick the winner of the decision (first
// minimum over the partial minima, or a forced id), report it and, if asked, make
// it s_i: state record, committed feature vector, running sums.
__global__ __launch_bounds__(64) void k_prepare(Tables t, int stage, uint32_t *decpack) {
  __shared__ DecPack pk;
  write_decpack(pk, t, blockIdx.x, stage, decpack);
}

__global__ __launch_bounds__(256) void k_commit(Tables t, int stage, int nparts, const float *pval,
                                               const int32_t *pidx, const int32_t *forced, int commit,
                                               uint32_t M, int32_t *best_cid, float *best_val,
                                               const uint32_t *decpack_cur, uint32_t *decpack_next) {
  __shared__ DecPack pk;
  Dec &d = pk.d;
  vf_space &sp = pk.sp;
  const int b = blockIdx.x, S = t.S, lane = threadIdx.x;
  if (decpack_cur) {
    // the decision's context was built for the scorer already: fetch it
    for (int i = lane; i < VF_DECPACK_DWORDS; i += (int)blockDim.x)
      reinterpret_cast<uint32_t *>(&pk)[i] = decpack_cur[(size_t)b * VF_DECPACK_DWORDS + i];
    __syncthreads();
  } else {
    build_dec(d, sp, t, b, stage);
  }
  // the decision's quotient tables, so that the one thread that evaluates the winner has no
  // chain of integer divisions to work through (built next to the reduction, by other waves)
  __shared__ EvalTabs tabs;
  fill_evaltabs(tabs, d, sp, 64);
  float v = __builtin_inff();
  int32_t c = -1;
  if (forced) {
    c = forced[(size_t)b * S + stage];
    v = 0.0f;
  } else if (lane < 64) {  // the first wave reduces the partial minima
    for (int p = lane; p < nparts; p += 64) {
      float pv = pval[(size_t)b * nparts + p];
      int32_t pi = pidx[(size_t)b * nparts + p];
      if (pi >= 0 && (pv < v || (pv == v && (c < 0 || pi < c)))) { v = pv; c = pi; }
    }
    for (int off = 32; off > 0; off >>= 1) {
      float ov = __shfl_down(v, off);
      int32_t oc = __shfl_down(c, off);
      if (oc >= 0 && (ov < v || (ov == v && (c < 0 || oc < c)))) { v = ov; c = oc; }
    }
  }
  __syncthreads();  // the tables are complete
  if (lane == 0) {
    if (best_cid) best_cid[b] = c;
    if (best_val) best_val[b] = v;
    if (commit) commit_winner(t, d, sp, b, stage, c, v, M, forced != nullptr, &tabs);
  }
  // the next stage's decision context, for the fused scorer
  if (commit && decpack_next && stage + 1 < S) {
    __threadfence();
    __syncthreads();
    write_decpack(pk, t, b, stage + 1, decpack_next);
  }
}

// ------------------------------------------------------------ beam search
//
// Secs. 3.1 and 4.1 also search with a beam guided by V, next to the greedy scan.
// The B problems of the context are the beam slots of one network.  Per layer: every
// live slot's candidates are scored (masked scores [B][Mpad]); the B smallest of all
// B*M scores survive, ordered by (score, parent slot, candidate id); survivor j copies
// its parent's schedule into slot j of the other table set and commits its candidate.

struct AltTables {
  int32_t *states, *cf, *prefix, *cids, *alive;
  float *vals;
};

__device__ __forceinline__ void take_min_u(float &v, int32_t &c, float ov, int32_t oc) {
  if (oc >= 0 && (ov < v || (ov == v && (c < 0 || oc < c)))) { v = ov; c = oc; }
}

// block-wide first minimum of (v, c); every thread gets the result
__device__ void block_min(float &v, int32_t &c, float *sv, int32_t *sc) {
  for (int off = 32; off > 0; off >>= 1) {
    float ov = __shfl_down(v, off);
    int32_t oc = __shfl_down(c, off);
    take_min_u(v, c, ov, oc);
  }
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sv[w] = v; sc[w] = c; }
  __syncthreads();
  v = sv[0]; c = sc[0];
  for (int k = 1; k < nw; ++k) take_min_u(v, c, sv[k], sc[k]);
}

// The same selection pass for a few survivors: k rounds of a block-wide first minimum
// (cheaper than sorting while k is small).
__global__ __launch_bounds__(256) void k_topk_pass_few(const float *val_in, const int32_t *idx_in, uint32_t n,
                                                   uint32_t M, uint32_t Mpad, int k, float *val_out,
                                                   int32_t *idx_out, int32_t *sel_n) {
  __shared__ float sv[4];
  __shared__ int32_t sc[4];
  const uint32_t base = blockIdx.x * 2048u;
  float v[8];
  int32_t id[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t i = base + threadIdx.x + e * 256u;
    float s = __builtin_inff();
    int32_t ix = -1;
    if (i < n) {
      if (idx_in) {
        ix = idx_in[i];
        if (ix >= 0) s = val_in[i];
      } else if ((i % Mpad) < M) {
        const float t = val_in[i];
        if (t < s) { s = t; ix = (int32_t)i; }  // NaN and +inf never survive
      }
    }
    v[e] = s;
    id[e] = ix;
  }
  int found = 0;
  for (int r = 0; r < k; ++r) {
    float bv = __builtin_inff();
    int32_t bi = -1;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (id[e] >= 0 && (v[e] < bv || (v[e] == bv && (bi < 0 || id[e] < bi)))) { bv = v[e]; bi = id[e]; }
    block_min(bv, bi, sv, sc);
    if (threadIdx.x == 0) {
      val_out[(size_t)blockIdx.x * k + r] = bv;
      idx_out[(size_t)blockIdx.x * k + r] = bi;
    }
    if (bi >= 0) {
      ++found;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (id[e] == bi) id[e] = -1;  // indices are unique: only the owner retires it
    }
  }
  if (sel_n && threadIdx.x == 0) {
    sel_n[0] = found;
    if (found > 0) sel_n[1] = found;
  }
}

// (value, index) as one sortable key: floats map to unsigned integers in their own order
// (-0 counts as +0, as in a comparison), the index breaks ties.  ~0 = no entry.
__device__ __forceinline__ unsigned long long topk_key(float v, int32_t idx) {
  uint32_t u = __float_as_uint(v == 0.0f ? 0.0f : v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (uint32_t)idx;
}
__device__ __forceinline__ float topk_value(unsigned long long key) {
  uint32_t u = (uint32_t)(key >> 32);
  u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
  return __uint_as_float(u);
}

// One selection pass: every block reduces 2048 (value, index) pairs to its k smallest,
// ordered by (value, index), with a bitonic sort of the keys in LDS.  First pass
// (idx_in == nullptr): values are the masked scores, index = slot * Mpad + candidate id,
// columns >= M are skipped.  Later passes read the pairs of the pass before.  The last
// pass (one block) also counts.  +inf and NaN never survive.
__global__ __launch_bounds__(256) void k_topk_pass(const float *val_in, const int32_t *idx_in, uint32_t n,
                                                   uint32_t M, uint32_t Mpad, int k, float *val_out,
                                                   int32_t *idx_out, int32_t *sel_n) {
  constexpr unsigned long long NONE = ~0ull;
  __shared__ unsigned long long keys[2048];
  const uint32_t base = blockIdx.x * 2048u;
  const int tid = threadIdx.x;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t i = base + tid + e * 256u;
    unsigned long long key = NONE;
    if (i < n) {
      if (idx_in) {
        const int32_t ix = idx_in[i];
        if (ix >= 0) key = topk_key(val_in[i], ix);
      } else if ((i % Mpad) < M) {
        const float t = val_in[i];
        if (t < __builtin_inff()) key = topk_key(t, (int32_t)i);
      }
    }
    keys[tid + e * 256] = key;
  }
  for (int size = 2; size <= 2048; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int t = tid + e * 256;
        const int lo = 2 * t - (t & (stride - 1)), hi = lo + stride;
        const bool up = (lo & size) == 0;
        const unsigned long long a = keys[lo], b = keys[hi];
        if ((a > b) == up) { keys[lo] = b; keys[hi] = a; }
      }
    }
  __syncthreads();
  for (int r = tid; r < k; r += 256) {
    const unsigned long long key = keys[r];
    val_out[(size_t)blockIdx.x * k + r] = key == NONE ? __builtin_inff() : topk_value(key);
    idx_out[(size_t)blockIdx.x * k + r] = key == NONE ? -1 : (int32_t)(uint32_t)key;
  }
  if (sel_n && tid == 0) {
    int found = 0;
    for (int r = 0; r < k; ++r) found += keys[r] != NONE;
    sel_n[0] = found;
    if (found > 0) sel_n[1] = found;
  }
}

// First layer of a beam search: only slot 0 (the context's current schedule of
// problem 0) is live; the other slots and the whole second table set are cleared.
__global__ __launch_bounds__(256) void k_beam_init(Tables t, AltTables alt, int B, int32_t *sel_n) {
  const int S = t.S;
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x, step = (size_t)gridDim.x * blockDim.x;
  const size_t n = (size_t)B * S;
  for (size_t i = i0; i < n * 64; i += step) { if (i >= (size_t)S * 64) t.cf[i] = 0; alt.cf[i] = 0; }
  for (size_t i = i0; i < n * 16; i += step) { if (i >= (size_t)S * 16) t.states[i] = 0; alt.states[i] = 0; }
  for (size_t i = i0; i < (size_t)B * (S + 1) * 2; i += step) { if (i >= (size_t)(S + 1) * 2) t.prefix[i] = 0; alt.prefix[i] = 0; }
  for (size_t i = i0; i < n; i += step) {
    if (i >= (size_t)S) { t.cids[i] = -1; t.vals[i] = __builtin_inff(); }
    alt.cids[i] = -1; alt.vals[i] = __builtin_inff();
  }
  for (size_t i = i0; i < (size_t)B; i += step) { t.alive[i] = (i == 0) ? t.alive[0] : 0; alt.alive[i] = 0; }
  if (i0 == 0) { sel_n[0] = 0; sel_n[1] = 1; }
}

// Survivor j of the layer: copy the parent's schedule, commit the candidate, build the
// next layer's decision context.  Slots past the survivors are cleared.  If nothing
// survived the schedules end: every slot is carried over unchanged and marked dead.
__global__ __launch_bounds__(64) void k_beam_commit(Tables t, AltTables nw, int stage, uint32_t M, uint32_t Mpad,
                                                    const float *sel_val, const int32_t *sel_idx, const int32_t *sel_n,
                                                    uint32_t *decpack_next) {
  __shared__ DecPack pk;
  const int j = blockIdx.x, S = t.S, lane = threadIdx.x;
  const int nsel = sel_n[0];
  const size_t dst = (size_t)j * S;
  int src_slot = -1;
  int32_t cid = -1;
  if (nsel == 0) src_slot = j;
  else if (j < nsel) { src_slot = sel_idx[j] / (int32_t)Mpad; cid = sel_idx[j] % (int32_t)Mpad; }
  const int rows = nsel == 0 ? S : stage;  // committed rows to carry over
  if (src_slot >= 0) {
    const size_t src = (size_t)src_slot * S;
    for (int i = lane; i < rows * 64; i += 64) nw.cf[dst * 64 + i] = t.cf[src * 64 + i];
    for (int i = lane; i < rows * 16; i += 64) nw.states[dst * 16 + i] = t.states[src * 16 + i];
    for (int i = lane; i < rows; i += 64) { nw.cids[dst + i] = t.cids[src + i]; nw.vals[dst + i] = t.vals[src + i]; }
    for (int i = lane; i < (S + 1) * 2; i += 64)
      nw.prefix[(size_t)j * (S + 1) * 2 + i] = (nsel == 0 || i < (stage + 1) * 2) ? t.prefix[(size_t)src_slot * (S + 1) * 2 + i] : 0;
  } else {
    for (int i = lane; i < (stage + 1) * 64; i += 64) nw.cf[dst * 64 + i] = 0;
    for (int i = lane; i < (stage + 1) * 16; i += 64) nw.states[dst * 16 + i] = 0;
    for (int i = lane; i <= stage; i += 64) { nw.cids[dst + i] = -1; nw.vals[dst + i] = __builtin_inff(); }
    for (int i = lane; i < (S + 1) * 2; i += 64) nw.prefix[(size_t)j * (S + 1) * 2 + i] = 0;
  }
  if (cid >= 0) {
    build_dec(pk.d, pk.sp, t, src_slot, stage);  // the parent's context, from the old tables
    if (lane == 0) {
      int32_t core[64];
      uint32_t dec;
      const bool ok = (uint32_t)cid < M && eval_candidate<true>(pk.d, pk.sp, (uint32_t)cid, dec, core);
      const size_t row = dst + stage;
      int32_t *pre = nw.prefix + ((size_t)j * (S + 1) + stage) * 2;
      if (ok) {
#pragma unroll
        for (int k = 0; k < 64; ++k) nw.cf[row * 64 + k] = core[k];
        int32_t *st = nw.states + row * 16;
        st[0] = core[17]; st[1] = core[18]; st[2] = core[19];
        st[3] = core[23]; st[4] = core[26]; st[5] = core[29]; st[6] = core[32]; st[7] = core[33];
        st[8] = core[34]; st[9] = core[35]; st[10] = core[36];
        st[11] = core[37];
        st[12] = core[20]; st[13] = core[21]; st[14] = core[22];
        st[15] = 1;
        nw.cids[row] = cid;
        nw.vals[row] = sel_val[j];
        pre[2] = sadd((uint32_t)pre[0], (uint32_t)core[40]);
        pre[3] = sadd((uint32_t)pre[1], (uint32_t)core[50]);
      } else {
        t.err[0] = 1;  // cannot happen: only valid candidates have finite scores
      }
      nw.alive[j] = ok ? 1 : 0;
    }
  } else if (lane == 0) {
    nw.alive[j] = 0;
  }
  if (decpack_next && stage + 1 < S) {
    __threadfence();
    __syncthreads();
    Tables tn = t;
    tn.states = nw.states; tn.cf = nw.cf; tn.prefix = nw.prefix; tn.cids = nw.cids; tn.alive = nw.alive; tn.vals = nw.vals;
    write_decpack(pk, tn, j, stage + 1, decpack_next);
  }
}

}  // namespace

int vfk_setup_tables(vf_ctx *c) {
  hipLaunchKernelGGL(k_setup, dim3(c->B), dim3(64), 0, c->stream, tables_of(c), c->d_intr, c->d_suffix);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

int vfk_rewind(vf_ctx *c, int first) {
  c->dec_stage = -1;
  hipLaunchKernelGGL(k_rewind, dim3((unsigned)c->B), dim3(256), 0, c->stream, tables_of(c), first);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

int vfk_reset_state(vf_ctx *c) {
  c->dec_stage = -1;
  size_t n = (size_t)c->B * c->S * 64;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_reset, dim3(blocks), dim3(256), 0, c->stream, tables_of(c), c->B);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

int vfk_enumerate(vf_ctx *c, int stage, uint32_t *dec, uint8_t *valid, int32_t *n_valid) {
  if (n_valid) {
    hipLaunchKernelGGL(k_fill_i32, dim3((c->B + 255) / 256), dim3(256), 0, c->stream, n_valid, (size_t)c->B, 0);
    VF_HIP(c, hipGetLastError());
  }
  dim3 grid((unsigned)(c->Mpad / 256), (unsigned)c->B);
  hipLaunchKernelGGL(k_enumerate, grid, dim3(256), 0, c->stream, tables_of(c), stage, (uint32_t)c->M,
                     (uint32_t)c->Mpad, dec, valid, n_valid);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

int vfk_featurize(vf_ctx *c, int stage, int32_t *feat) {
  vf_prof_scope prof(c, VF_PROF_FEATURIZE);
  dim3 grid((unsigned)((c->Mpad / 256 + VF_FEAT_SPAN - 1) / VF_FEAT_SPAN), (unsigned)c->B);
  hipLaunchKernelGGL(k_featurize, grid, dim3(256), 0, c->stream, tables_of(c), stage, (uint32_t)c->M,
                     (uint32_t)c->Mpad, (int)c->space.F, feat);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

int vfk_commit_from_partials(vf_ctx *c, int stage, int nparts, int commit, int32_t *best_cid, float *best_val) {
  vf_prof_scope prof(c, VF_PROF_COMMIT);
  hipLaunchKernelGGL(k_commit, dim3(c->B), dim3(256), 0, c->stream, tables_of(c), stage, nparts, c->d_pval,
                     c->d_pidx, (const int32_t *)nullptr, commit, (uint32_t)c->M, best_cid, best_val,
                     c->dec_stage == stage ? (const uint32_t *)c->d_decpack : (const uint32_t *)nullptr, c->d_decpack);
  VF_HIP(c, hipGetLastError());
  if (commit) c->dec_stage = stage + 1 < c->S ? stage + 1 : -1;
  return VF_OK;
}

int vfk_commit_from(vf_ctx *c, int stage, int nparts, const float *pval, const int32_t *pidx, const uint32_t *decpack_cur) {
  vf_prof_scope prof(c, VF_PROF_COMMIT);
  hipLaunchKernelGGL(k_commit, dim3(c->B), dim3(256), 0, c->stream, tables_of(c), stage, nparts, pval, pidx,
                     (const int32_t *)nullptr, 1, (uint32_t)c->M, (int32_t *)nullptr, (float *)nullptr, decpack_cur,
                     c->d_decpack);
  VF_HIP(c, hipGetLastError());
  c->dec_stage = stage + 1 < c->S ? stage + 1 : -1;
  return VF_OK;
}

int vfk_commit_forced(vf_ctx *c, int stage) {
  hipLaunchKernelGGL(k_commit, dim3(c->B), dim3(256), 0, c->stream, tables_of(c), stage, 0,
                     (const float *)nullptr, (const int32_t *)nullptr, (const int32_t *)c->d_forced, 1,
                     (uint32_t)c->M, (int32_t *)nullptr, (float *)nullptr, (const uint32_t *)nullptr,
                     (uint32_t *)nullptr);
  VF_HIP(c, hipGetLastError());
  c->dec_stage = -1;
  return VF_OK;
}

int vfk_prepare(vf_ctx *c, int stage) {
  if (c->dec_stage == stage) return VF_OK;
  hipLaunchKernelGGL(k_prepare, dim3(c->B), dim3(64), 0, c->stream, tables_of(c), stage, c->d_decpack);
  VF_HIP(c, hipGetLastError());
  c->dec_stage = stage;
  return VF_OK;
}

static int beam_alloc(vf_ctx *c) {
  if (c->d_alt_states) return VF_OK;
  const size_t n = (size_t)c->S * c->B;
  struct { void **p; size_t bytes; } want[] = {
      {(void **)&c->d_alt_states, n * 16 * 4}, {(void **)&c->d_alt_cf, n * 64 * 4},
      {(void **)&c->d_alt_prefix, (size_t)c->B * (c->S + 1) * 2 * 4}, {(void **)&c->d_alt_cids, n * 4},
      {(void **)&c->d_alt_vals, n * 4}, {(void **)&c->d_alt_alive, (size_t)c->B * 4},
      {(void **)&c->d_sel_val, (size_t)c->B * 4}, {(void **)&c->d_sel_idx, (size_t)c->B * 4},
      {(void **)&c->d_sel_n, 2 * 4}};
  for (auto &w : want) {
    if (*w.p) continue;
    if (hipMalloc(w.p, w.bytes ? w.bytes : 4) != hipSuccess) { (void)hipGetLastError(); return VF_ENOMEM; }
  }
  return VF_OK;
}

static AltTables alt_of(const vf_ctx *c) {
  AltTables a;
  a.states = c->d_alt_states; a.cf = c->d_alt_cf; a.prefix = c->d_alt_prefix; a.cids = c->d_alt_cids;
  a.alive = c->d_alt_alive; a.vals = c->d_alt_vals;
  return a;
}

int vfk_beam_init(vf_ctx *c, int first_stage) {
  (void)first_stage;
  int rc = beam_alloc(c);
  if (rc != VF_OK) return rc;
  size_t n = (size_t)c->B * c->S * 64;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_beam_init, dim3(blocks), dim3(256), 0, c->stream, tables_of(c), alt_of(c), c->B, c->d_sel_n);
  VF_HIP(c, hipGetLastError());
  c->dec_stage = -1;
  return VF_OK;
}

// scores of the layer are in d_scores: select the survivors, commit them into the other
// table set, swap the sets
int vfk_beam_select_commit(vf_ctx *c, int stage) {
  const uint32_t total = (uint32_t)((size_t)c->B * c->Mpad);
  const int nchunks = (int)((total + 2047u) / 2048u), k = c->B;
  const size_t want = (size_t)nchunks * k;
  if (want > c->tk_elems) {
    if (c->d_tk_val) { VF_HIP(c, hipStreamSynchronize(c->stream)); (void)hipFree(c->d_tk_val); (void)hipFree(c->d_tk_idx); }
    c->d_tk_val = nullptr; c->d_tk_idx = nullptr; c->tk_elems = 0;
    if (hipMalloc((void **)&c->d_tk_val, want * 8) != hipSuccess || hipMalloc((void **)&c->d_tk_idx, want * 8) != hipSuccess) {
      (void)hipGetLastError();
      return VF_ENOMEM;
    }
    c->tk_elems = want;
  }
  // passes of 2048 -> k until one block is left; buffers alternate between the two halves
  float *va = c->d_tk_val, *vb = c->d_tk_val + want;
  int32_t *ia = c->d_tk_idx, *ib = c->d_tk_idx + want;
  const float *vin = c->d_scores;
  const int32_t *iin = nullptr;
  uint32_t n = total;
  for (;;) {
    const int blocks = (int)((n + 2047u) / 2048u);
    const bool last_pass = blocks == 1;
    hipLaunchKernelGGL(k <= 16 ? k_topk_pass_few : k_topk_pass, dim3(blocks), dim3(256), 0, c->stream, vin, iin, n, (uint32_t)c->M,
                       (uint32_t)c->Mpad, k, last_pass ? c->d_sel_val : va, last_pass ? c->d_sel_idx : ia,
                       last_pass ? c->d_sel_n : (int32_t *)nullptr);
    VF_HIP(c, hipGetLastError());
    if (last_pass) break;
    vin = va; iin = ia;
    n = (uint32_t)blocks * (uint32_t)k;
    std::swap(va, vb);
    std::swap(ia, ib);
  }
  {
    vf_prof_scope prof(c, VF_PROF_COMMIT);
    hipLaunchKernelGGL(k_beam_commit, dim3(c->B), dim3(64), 0, c->stream, tables_of(c), alt_of(c), stage,
                       (uint32_t)c->M, (uint32_t)c->Mpad, c->d_sel_val, c->d_sel_idx, c->d_sel_n, c->d_decpack);
    VF_HIP(c, hipGetLastError());
  }
  std::swap(c->d_states, c->d_alt_states);
  std::swap(c->d_cf, c->d_alt_cf);
  std::swap(c->d_prefix, c->d_alt_prefix);
  std::swap(c->d_cids, c->d_alt_cids);
  std::swap(c->d_vals, c->d_alt_vals);
  std::swap(c->d_alive, c->d_alt_alive);
  c->dec_stage = stage + 1 < c->S ? stage + 1 : -1;
  return VF_OK;
}
