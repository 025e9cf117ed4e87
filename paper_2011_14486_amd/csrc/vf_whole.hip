// Algorithm 1 for whole problems in one launch (gfx950): a workgroup (or a team of
// workgroups) owns a problem from its first undecided stage to the last and does every
// step of the greedy scan by itself - decision context, the list of valid candidates,
// their features, V(s) with the bf16 MLP, the running minimum, the commit "s_i := s" -
// so that a schedule costs one launch and nothing but the tables and the id list touches
// memory.  Used from 24 problems on (below that the two launches per layer are faster).
//
// The MLP is the same contraction as in the per-layer scorer: weights are the MFMA A
// operand and stream from L2 through a ring of registers, activations are the B operand
// in LDS, a wave owns RT row tiles of every hidden layer and all NC / 32 column tiles.
// What differs is the tile pipeline.  The features of a tile (rows 16..63 of the input; all
// other rows are the same for all candidates of a decision and enter as a bias, see below)
// go to an input buffer of their own, so the first layer does not have to share the
// activation buffer with the layers behind it, and they are produced one tile ahead:
// waves 4..7 evaluate the next tile's candidates before their share of the last hidden
// layer and waves 0..3 after it, so that on every SIMD one wave's integer work runs under
// the other wave's matrix work.  The scan over a tile's scores is left to the waves that
// hold them while the others start the next tile.  Two workgroup barriers per tile remain:
// one behind the first layer's activations, one behind the partial output dots.
#include <stdlib.h>

#include "vf_internal.h"

namespace {

#include "vf_sched_dev.h"

#include "vf_score_dev.h"

// With fewer problems than compute units a team of `team` workgroups shares one problem:
// every member builds the decision's context and id list for itself, member m scores
// tiles m, m + team, ... of the list, publishes its minimum, the team meets at a counter
// in global memory (one arrival per member and layer, bounded wait), and every member then
// reduces all minima and commits by itself - the members write identical values to the
// tables and the list, so one meeting per layer is enough.
//
// With more problems than half the compute units (team = 1) the problems differ in size,
// and the launch would take as long as the largest one.  Then a workgroup that has
// finished its own problems (or never had one) becomes a helper: it queues up in a pool.
// An owner that starts a layer with enough tiles takes up to VF_MAX_HELPERS workgroups out
// of the pool and sends each of them the layer (problem, layer, team size, member index)
// through its mailbox; the helper fetches what the owner has worked out for the layer and
// left in memory (decision context, quotient tables, folded bias, the candidate list),
// scores tiles member, member + team, ..., publishes its minimum, reports its arrival and
// queues up again - it neither waits for anybody nor commits.  The owner waits (bounded) for the arrivals of the helpers it sent for and commits
// alone.  The grid is one workgroup per compute unit, so every workgroup that is waited
// for is resident; helpers leave when every problem is done.
struct WholeArgs {
  Tables t;
  int first, last;
  uint32_t *list;  // [nprob][Mpad] scratch for the lists of valid candidates (their packed digits)
  int64_t Mpad;
  int team;                  // workgroups per problem; grid = nprob * team <= compute units when > 1
  int helpers;               // team == 1: idle workgroups help (grid = compute units)
  int tstride;               // slots per problem in team_val / team_idx
  float *team_val;           // [2][nprob][tstride] per-member minima, by layer parity
  int32_t *team_idx;
  unsigned int *team_count;  // [nprob] arrivals at the meetings, zero at launch
  int32_t *team_err;         // set if a wait ran out
  unsigned int wait_rounds;  // polling rounds after which a wait gives up
  // the pool (all zero at launch)
  unsigned int *pool;                // [0] entries taken, [1] entries put, [2] problems done
  unsigned int *pool_q;              // [VF_POOL_SLOTS] workgroup id + 1 of a queued helper, 0 = empty
  unsigned long long *mailbox;       // [grid] the layer a helper is sent: see mail_pack
  uint32_t *pub;                     // [nprob][VF_PUB_WORDS] what an owner leaves for its helpers: the layer's
                                     // decision context, quotient tables, folded bias and candidate count
};
// words of an owner's published layer: DecPack, EvalTabs, first-layer bias (up to 1024 rows), count
constexpr int VF_PUB_TABS = VF_DECPACK_DWORDS;
constexpr int VF_PUB_BIAS = VF_PUB_TABS + (int)(sizeof(EvalTabs) / 4);
constexpr int VF_PUB_COUNT = VF_PUB_BIAS + 1024;
constexpr int VF_PUB_WORDS = VF_PUB_COUNT + 4;
constexpr int VF_XIN_STRIDE = 56;  // elements between the columns of the input buffer (48 used)
constexpr int VF_MAX_HELPERS = 3;
constexpr int VF_POOL_SLOTS = 1024;       // more than the workgroups of a launch
constexpr int VF_TILES_PER_MEMBER = 4;    // a helper is sent for when every member gets at least this many tiles

// What a mailbox holds: never zero (zero = empty).
__device__ __forceinline__ unsigned long long mail_pack(int unit, int stage, int team, int member) {
  return 1ull << 63 | (unsigned long long)unit << 40 | (unsigned long long)stage << 16 |
         (unsigned long long)team << 8 | (unsigned long long)member;
}

// NC candidates per tile, RT row tiles per wave (hidden width 256 * RT), PD k-steps of
// weight fragments in flight per wave.  stat: nullable, [0] += candidates pushed through
// the network, [1] += valid ones (the same here: only valid ids are listed).
// ONE: the network has a single hidden layer (otherwise two).
template <int NC, int RT, int PD, bool ONE>
__global__ __launch_bounds__(512) void k_whole(vf_fast_dev md, int ks, int64_t M, int nprob,
                                               unsigned long long *stat, NoiseArgs na, WholeArgs wa) {
  constexpr int CT = NC / 32;
  constexpr int NWS = NC / 64;  // waves that scan the tile's scores: wave w owns columns 64 w ...
  constexpr int XS = VF_XIN_STRIDE;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *act = reinterpret_cast<uint16_t *>(smem);          // [NC][ks] hidden activations
  uint16_t *xin = act + (size_t)NC * ks;                       // [NC][XS] rows 16..63 of the tile's candidates
                                                               // (48 values, columns 112 bytes apart)
  float *red = reinterpret_cast<float *>(xin + (size_t)NC * XS);  // [8][NC] partial output dots
  int32_t *okf = reinterpret_cast<int32_t *>(red + 8 * NC);    // [2][NC] candidate id + 1 of a valid column, else 0
  float *auxs = reinterpret_cast<float *>(okf + 2 * NC);       // biases; output vector as bfloat16 pairs
  __shared__ DecPack pk;
  __shared__ EvalTabs tabs;  // the decision's quotient tables: no division per candidate
  __shared__ int team_failed;
  __shared__ float sv[NWS];      // per scanning wave: the minimum over its columns at the end of a layer
  __shared__ int32_t sc[NWS];
  __shared__ unsigned int sn[2];  // what the layer counted (candidates, valid ones)
  // Only rows 16..55 and 59 of the network's input depend on the candidate; the part of the
  // first layer that belongs to all the other rows (intrinsic block, context rows, with 256
  // inputs the neighbour stages) is a per-decision bias, which replaces the layer's bias in
  // LDS, and the contraction runs over rows 16..63 with zeros in the shared rows among them

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int NH = md.L - 1;

  // ---- once per workgroup: the small fp32 vectors into LDS, the weight ring primed
  // (the output vector's values are bfloat16 numbers: two to a word, to save LDS)
  for (int i = tid; i < (int)md.wl_off; i += 512) auxs[i] = md.aux[i];
  for (int i = tid; i < md.dims[NH] / 2; i += 512)
    reinterpret_cast<uint32_t *>(auxs + md.wl_off)[i] = pack_bf16(md.aux[md.wl_off + 2 * i], md.aux[md.wl_off + 2 * i + 1]);
  const __amdgpu_buffer_rsrc_t ws = stream_rsrc(md.w_stream + (size_t)w * md.wave_stride);
  const __amdgpu_buffer_rsrc_t wf = stream_rsrc(md.w_full + (size_t)w * md.wave_stride_full);
  const int voff = 16 * lane;
  int wstep = 0;
  uint4 ring[PD][RT];
#pragma unroll
  for (int j = 0; j < PD; ++j)
#pragma unroll
    for (int r = 0; r < RT; ++r) ring[j][r] = stream_load(ws, voff, j * RT + r);

  if (tid == 0) team_failed = 0;
  // what this workgroup does next: a layer of one of its own problems (owner), or a layer it
  // is sent as a helper.  Thread 0 finds out and hands the result to the others through LDS.
  __shared__ int job_unit, job_stage, job_team, job_member;
  bool helping = false;
  int unit = (int)blockIdx.x / wa.team, stage = wa.first;
  unsigned int owner_target = 0u;  // thread 0, owner: helper arrivals the problem's layers so far sent for
  for (;;) {
    int team = wa.team, member = (int)blockIdx.x % wa.team;
    if (!helping && unit >= nprob) {
      if (!wa.helpers) break;
      helping = true;
    }
    if (helping) {
      // queue up in the pool, then wait for mail (bounded) or for every problem to be done
      if (tid == 0) {
        job_stage = -1;
        const unsigned int slot = atomicAdd(&wa.pool[1], 1u);
        __hip_atomic_store(&wa.pool_q[slot % VF_POOL_SLOTS], (unsigned int)blockIdx.x + 1u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        // (the bound counts rounds without any problem finishing anywhere: a launch that is merely
        // long - very many problems, a GPU shared with other work - does not run it out)
        unsigned int spins = 0, seen_done = 0;
        for (;;) {
          const unsigned long long m = __hip_atomic_load(&wa.mailbox[blockIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (m != 0ull) {
            job_unit = (int)((m >> 40) & 0x7fffffull); job_stage = (int)((m >> 16) & 0xffffffull);
            job_team = (int)((m >> 8) & 255ull); job_member = (int)(m & 255ull);
            // emptied before this workgroup queues up again
            __hip_atomic_store(&wa.mailbox[blockIdx.x], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          const unsigned int done = __hip_atomic_load(&wa.pool[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (done >= (unsigned int)nprob) break;
          if (done != seen_done) { seen_done = done; spins = 0; }
          if (++spins > wa.wait_rounds) { team_failed = 1; wa.team_err[0] = 1; break; }
          __builtin_amdgcn_s_sleep(8);
        }
        __threadfence();  // what the owner wrote before it sent the mail is read from memory
      }
      __syncthreads();
      if (team_failed) return;
      if (job_stage < 0) break;  // every problem is done
      unit = job_unit; stage = job_stage; team = job_team; member = job_member;
    }
    uint32_t *const idlist = wa.list + (size_t)unit * wa.Mpad;
    na.stage = stage;
    __shared__ int ncand, g_npairs;
    __shared__ unsigned int job_helper[VF_MAX_HELPERS];
    uint32_t *const pub = wa.pub + (size_t)unit * VF_PUB_WORDS;
    if (helping) {
      // the owner has left the layer in memory before it sent the mail
      for (int i = tid; i < VF_DECPACK_DWORDS; i += 512) reinterpret_cast<uint32_t *>(&pk)[i] = pub[i];
      for (int i = tid; i < (int)(sizeof(EvalTabs) / 4); i += 512) reinterpret_cast<uint32_t *>(&tabs)[i] = pub[VF_PUB_TABS + i];
      for (int i = tid; i < md.dims[1]; i += 512) auxs[md.bias_off[0] + i] = __uint_as_float(pub[VF_PUB_BIAS + i]);
      if (tid == 0) ncand = (int)pub[VF_PUB_COUNT];
      __syncthreads();
    } else {
    build_dec(pk.d, pk.sp, wa.t, unit, stage);
    // three small jobs side by side, on different waves: the quotient tables (waves 0, 1), the
    // shared input rows as the first layer wants them (waves 2, 3), the split factors that fit
    // (wave 4)
    fill_evaltabs(tabs, pk.d, pk.sp);
    if (tid >= 128 && tid < 128 + VF_STAT_WORDS) pk.stat[tid - 128] = stat_word(pk.d, tid - 128);
    // Ordered list of the decision's valid ids, written down directly from the validity
    // rules: per (compute_at, store_at) digit pair that is open - the level is offered and
    // the hoist does not exceed it - the valid ids are the products of the split factors
    // that fit the level's region with every loop order / vectorize / parallel choice;
    // an inlining pair has the single id with every other digit zero.  The list holds the
    // digits, packed, rather than the id: the evaluation works on digits, and putting an id
    // together takes a few multiplications where taking it apart takes as many divisions.
    __shared__ int g_pos[13], g_cat[12], g_dec[12];
    __shared__ int g_nok[3][3], g_ok[3][3][8];
    __shared__ float g_rcp[3][3];  // 1 / g_nok, for div_small
    if (tid >= 256 && tid < 265) {
      const int lvl = (tid - 256) / 3, dd = (tid - 256) % 3;
      int cnt = 0;
      for (int k = 0; k < pk.sp.nf[dd]; ++k)
        if ((uint32_t)pk.sp.fac[dd][k] <= pk.d.E[lvl][dd]) g_ok[lvl][dd][cnt++] = k;
      g_nok[lvl][dd] = cnt;
      g_rcp[lvl][dd] = 1.0f / (float)(cnt > 0 ? cnt : 1);
    }
    __syncthreads();
    const int rest_n = pk.sp.nperm * pk.sp.nvec * pk.sp.npar;
    const float rcp_perm = 1.0f / (float)pk.sp.nperm, rcp_vec = 1.0f / (float)pk.sp.nvec;
    if (w == 0) {
      // lane j looks at pair j = (store_at digit, compute_at digit); the open pairs are then
      // numbered and given their first list position in order
      const int npairs_all = pk.sp.nsat * pk.sp.ncat;
      int cnt = 0, cat = 0, dec = 0;
      if (lane < npairs_all && lane < 12) {
        const int isat = lane / pk.sp.ncat, icat = lane % pk.sp.ncat;
        cat = pk.sp.cat[icat];
        dec = (int)((uint32_t)icat << 24 | (uint32_t)isat << 28);
        if (pk.d.lvl_ok[cat] != 0) {
          if (cat == VF_INLINE) cnt = isat == 0 ? 1 : 0;
          else if (isat <= cat) cnt = g_nok[cat][0] * g_nok[cat][1] * g_nok[cat][2] * rest_n;
        }
      }
      int np = 0, pos = 0;
#pragma unroll
      for (int j = 0; j < 12; ++j) {
        const int cj = __builtin_amdgcn_readlane(cnt, j);
        if (cj == 0) continue;
        const int catj = __builtin_amdgcn_readlane(cat, j), decj = __builtin_amdgcn_readlane(dec, j);
        if (lane == 0) {
          g_pos[np] = pos;
          g_cat[np] = catj;
          g_dec[np] = decj;
        }
        pos += cj;
        ++np;
      }
      if (lane == 0) {
        g_pos[np] = pos;
        g_npairs = np;
        ncand = pos;
      }
    }
    fold_bias<RT>(wf, pk.stat, md.dims[0] == 256, w, lane,
                  md.aux + md.bias_off[0], auxs + md.bias_off[0]);
    __syncthreads();  // the pairs are numbered, the bias is complete
    // (the pairs' first positions into registers: the pair of an entry is then found without
    // a chain of dependent reads)
    int pos_r[12];
#pragma unroll
    for (int j = 0; j < 12; ++j) pos_r[j] = j < g_npairs ? g_pos[j] : 0x7fffffff;
    for (int k = tid; k < ncand; k += 512) {
      int q = 0;
#pragma unroll
      for (int j = 1; j < 12; ++j) q += k >= pos_r[j] ? 1 : 0;
      const int cat = g_cat[q];
      uint32_t dec = (uint32_t)g_dec[q];
      if (cat != VF_INLINE) {
        uint32_t r = (uint32_t)(k - g_pos[q]), nxt;
        const uint32_t nx = g_nok[cat][0], ny = g_nok[cat][1], nc = g_nok[cat][2];
        nxt = div_small(r, nx, g_rcp[cat][0]); const uint32_t jx = r - nxt * nx; r = nxt;
        nxt = div_small(r, ny, g_rcp[cat][1]); const uint32_t jy = r - nxt * ny; r = nxt;
        nxt = div_small(r, nc, g_rcp[cat][2]); const uint32_t jc = r - nxt * nc; r = nxt;
        const int ix = g_ok[cat][0][jx], iy = g_ok[cat][1][jy], ic = g_ok[cat][2][jc];
        nxt = div_small(r, (uint32_t)pk.sp.nperm, rcp_perm); const uint32_t ip = r - nxt * (uint32_t)pk.sp.nperm; r = nxt;
        const uint32_t par = div_small(r, (uint32_t)pk.sp.nvec, rcp_vec), vec = r - par * (uint32_t)pk.sp.nvec;
        dec |= (uint32_t)ix | (uint32_t)iy << 4 | (uint32_t)ic << 8 | (uint32_t)ip << 12 | (uint32_t)vec << 16 |
               (uint32_t)par << 20;
      }
      idlist[k] = dec;
    }
    if (wa.helpers) {
      // owner: with enough tiles, up to VF_MAX_HELPERS workgroups are taken out of the pool
      if (tid == 0) {
        int n = 0;
        int want = (ncand + NC - 1) / NC / VF_TILES_PER_MEMBER - 1;
        if (want > VF_MAX_HELPERS) want = VF_MAX_HELPERS;
        for (int attempt = 0; attempt < 4 && want > 0 && n == 0; ++attempt) {
          const unsigned int taken = __hip_atomic_load(&wa.pool[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const int avail = (int)(__hip_atomic_load(&wa.pool[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - taken);
          if (avail <= 0) break;
          const int take = avail < want ? avail : want;
          if (atomicCAS(&wa.pool[0], taken, taken + (unsigned int)take) != taken) continue;  // somebody else took some
          for (int i = 0; i < take; ++i) {
            unsigned int *const q = &wa.pool_q[(taken + (unsigned int)i) % VF_POOL_SLOTS];
            unsigned int id = 0u, spins = 0u;
            // (the helper bumps the count before it writes its id)
            while ((id = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == 0u) {
              if (++spins > wa.wait_rounds) { team_failed = 1; wa.team_err[0] = 1; break; }
              __builtin_amdgcn_s_sleep(1);
            }
            if (id == 0u) break;
            __hip_atomic_store(q, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            job_helper[i] = id - 1u;
          }
          n = take;
        }
        job_team = 1 + n;
        owner_target += (unsigned int)n;
      }
    }
    }  // (not helping)
    __syncthreads();  // the id list (written by this workgroup) is complete
    if (team_failed) return;
    if (wa.helpers && !helping) {
      team = job_team;
      if (team > 1) {
        // what a helper needs of this layer goes to memory (the list is there already); the
        // helpers are sent for once all of it has arrived: every thread waits for its own
        // stores, then thread 0 sends the mail
        for (int i = tid; i < VF_DECPACK_DWORDS; i += 512) pub[i] = reinterpret_cast<const uint32_t *>(&pk)[i];
        for (int i = tid; i < (int)(sizeof(EvalTabs) / 4); i += 512) pub[VF_PUB_TABS + i] = reinterpret_cast<const uint32_t *>(&tabs)[i];
        for (int i = tid; i < md.dims[1]; i += 512) pub[VF_PUB_BIAS + i] = __float_as_uint(auxs[md.bias_off[0] + i]);
        if (tid == 0) pub[VF_PUB_COUNT] = (uint32_t)ncand;
        __threadfence();
        __syncthreads();
        if (tid == 0)
          for (int i = 0; i + 1 < team; ++i)
            __hip_atomic_store(&wa.mailbox[job_helper[i]], mail_pack(unit, stage, team, i + 1), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    const int ncands = ncand;
    const int ntiles = (ncands + NC - 1) / NC;

    // Thread tid evaluates the candidate of column tid % NC of the tile that starts at list
    // entry nb and stores its share of rows 16..63, normalised, as bf16 (8 rows = one 16-byte
    // chunk): part 0 rows 16..31, part 1 rows 32..39 and 56..63 (of which only row 59 is the
    // candidate's own: the others belong to the bias and stay zero), part 2 rows 40..47, part
    // 3 rows 48..55 - dealt out so that the four copies cost about the same; the rows a part
    // does not store are dead code in its copy of the evaluation.  Padding columns evaluate id
    // 0 and store zeros.
    auto featurize = [&](int nb, int par) __attribute__((always_inline)) {
      const int n = tid % NC, part = tid / NC;
      const bool inb = (nb + n) < ncands;
      const Digits dg = unpack_digits(inb ? idlist[nb + n] : 0u);
      int32_t core[64];
      uint16_t *const col = xin + (size_t)n * XS;
      auto put8 = [&](const int32_t *v, int chunk) {
        uint4 q;
        q.x = pack_bf16(plog2_dev(v[0]), plog2_dev(v[1]));
        q.y = pack_bf16(plog2_dev(v[2]), plog2_dev(v[3]));
        q.z = pack_bf16(plog2_dev(v[4]), plog2_dev(v[5]));
        q.w = pack_bf16(plog2_dev(v[6]), plog2_dev(v[7]));
        if (!inb) q = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4 *>(col + (chunk << 3)) = q;
      };
      if (part == 0) {
        // evaluated for padding ids too: core must be defined before it is packed
        const bool valid = eval_digits<true>(pk.d, pk.sp, dg, &tabs, core);
        okf[par * NC + n] = (inb && valid) ? (int32_t)id_of(pk.sp, dg) + 1 : 0;
        put8(core + 16, 0);
        put8(core + 24, 1);
      } else if (part == 1) {
        eval_digits<true>(pk.d, pk.sp, dg, &tabs, core);
        put8(core + 32, 2);
        *reinterpret_cast<uint4 *>(col + 40) = make_uint4(0u, inb ? pack_bf16(0.0f, plog2_dev(core[59])) : 0u, 0u, 0u);
      } else if (part == 2) {
        eval_digits<true>(pk.d, pk.sp, dg, &tabs, core);
        put8(core + 40, 3);
      } else if (part == 3) {
        eval_digits<true>(pk.d, pk.sp, dg, &tabs, core);
        put8(core + 48, 4);
      }
    };

    // Waves below NWS scan the scores: thread tid keeps the incumbent of column tid over the
    // tiles of the layer (and counts, candidates in the low half, valid ones in the high half),
    // the columns are reduced once per layer.  Behind the barrier that ends a tile these
    // threads only add up their column's partial dots; the rest of the scan - noise, the
    // comparison with the incumbent - waits until they have nothing else to do: the end of
    // their part of the next tile, where they would otherwise wait for the other waves.
    float col_v = __builtin_inff();
    int32_t col_c = -1;
    unsigned int col_n = 0u;
    float pend_s = 0.0f;     // a tile's score of this thread's column that has not been scanned yet
    int32_t pend_flag = -1;  // its candidate id + 1, 0 = not a valid column, -1 = nothing pending
    auto scan_pending = [&]() __attribute__((always_inline)) {
      if (pend_flag < 0) return;
      float sv_ = pend_s;
      const int32_t colid = pend_flag - 1;
      if (pend_flag != 0) {
        if (na.eps != 0.0f) sv_ = add_noise(na, sv_, unit, colid);
        // (+inf and NaN never win: Algorithm 1 compares with a strict "<" from +inf)
        if (sv_ < __builtin_inff()) take_min(col_v, col_c, sv_, colid);
      }
      pend_flag = -1;
    };
    if (tid == 0) sn[0] = sn[1] = 0u;
    const uint16_t *const bx = xin + (size_t)(lane & 31) * XS + 8 * (lane >> 5);
    const uint16_t *const ba = act + (size_t)(lane & 31) * ks + 8 * (lane >> 5);
    // a hidden layer's output becomes the next one's input: rounded to bfloat16, ReLU on the
    // pairs; the two lane halves then trade their row groups so that every lane writes 8
    // consecutive rows of its column at once
    auto write_back = [&](floatx16 (&acc)[RT][CT]) __attribute__((always_inline)) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        const int m0 = (w + r * 8) * 32 + 8 * (lane >> 5);
#pragma unroll
        for (int g = 0; g < 4; g += 2) {
#pragma unroll
          for (int c = 0; c < CT; ++c) {
            uint32_t x0 = relu_bf16x2(pack_bf16(acc[r][c][4 * g + 0], acc[r][c][4 * g + 1]));
            uint32_t x1 = relu_bf16x2(pack_bf16(acc[r][c][4 * g + 2], acc[r][c][4 * g + 3]));
            uint32_t y0 = relu_bf16x2(pack_bf16(acc[r][c][4 * g + 4], acc[r][c][4 * g + 5]));
            uint32_t y1 = relu_bf16x2(pack_bf16(acc[r][c][4 * g + 6], acc[r][c][4 * g + 7]));
            swap_halves(x0, y0);
            swap_halves(x1, y1);
            *reinterpret_cast<uint4 *>(act + (size_t)(c * 32 + (lane & 31)) * ks + m0 + 8 * g) = make_uint4(x0, x1, y0, y1);
          }
        }
      }
    };
    // the last hidden layer is never written back: rounded to bf16, it is multiplied with the
    // output vector at once
    auto output_dots = [&](floatx16 (&acc)[RT][CT], float (&dot)[CT]) __attribute__((always_inline)) {
      const uint32_t *wl = reinterpret_cast<const uint32_t *>(auxs + md.wl_off);
      output_dots_mfma<RT, CT>(acc, dot, [&](int u) { return wl[u >> 1]; }, w, lane);
    };

    // the loop starts one tile early: that round only produces the first tile's features
    int par = 1;
    for (int t = member - team; t < ntiles; t += team, par ^= 1) {
      const bool real = t >= member;
      const bool has_next = t + team < ntiles;
      float dot[CT];
      // ---- first layer, over the candidates' own rows in the input buffer.  (The matrix
      // loops go first on their SIMD: the other wave's vector work fills the gaps.)
      if constexpr (ONE) {
        // a single hidden layer: its output goes straight into the output dots; the next
        // tile's features land in the buffer that the layer has read, so every wave finishes
        // the layer first
        if (real) {
          floatx16 acc[RT][CT], bv[RT];
          load_bias<RT>(bv, auxs + md.bias_off[0], w, lane);
          __builtin_amdgcn_s_setprio(2);
          contract_own_rows<RT, CT, PD, true>(acc, bv, ring, ws, voff, bx, 32 * XS);
          __builtin_amdgcn_s_setprio(0);
          output_dots(acc, dot);
        }
        __syncthreads();
        if (has_next) featurize((t + team) * NC, par ^ 1);
      } else {
        if (real) {
          floatx16 acc[RT][CT], bv[RT];
          load_bias<RT>(bv, auxs + md.bias_off[0], w, lane);
          __builtin_amdgcn_s_setprio(2);
          contract_own_rows<RT, CT, PD, false>(acc, bv, ring, ws, voff, bx, 32 * XS);
          __builtin_amdgcn_s_setprio(0);
          wstep = VF_K0_OWN + PD;
          // (nobody reads the activations of the tile before any more: barrier behind its dots)
          write_back(acc);
          __syncthreads();
        }
        // ---- last hidden layer and the output dots; the next tile's features.  Waves 4..7
        // produce their share of the features before the layer, waves 0..3 after it, so that
        // on every SIMD one wave's integer work runs under the other wave's matrix work.  The
        // last PD steps of the contraction prefetch the first PD steps of the next tile.
        for (int ph = 0; ph < 2; ++ph) {
          if ((ph == 0) == (w >= 4)) {
            if (has_next) featurize((t + team) * NC, par ^ 1);
            continue;
          }
          if (!real) continue;
          floatx16 acc[RT][CT], bv[RT];
          load_bias<RT>(bv, auxs + md.bias_off[1], w, lane);
          __builtin_amdgcn_s_setprio(2);
          contract_layer<RT, CT, PD, VF_K0_OWN % PD>(acc, bv, ring, ws, wstep, voff, true, md.dims[1] / 16, ba, 32 * ks);
          __builtin_amdgcn_s_setprio(0);
          output_dots(acc, dot);
        }
      }
      // the scan of the tile before, by the waves that hold its scores (nothing left to do
      // for them before the barrier)
      if (w < NWS) scan_pending();

      // ---- value: the waves' parts of the dots (lanes 0..31 hold them), summed in order behind the barrier
      if (real) {
#pragma unroll
        for (int c = 0; c < CT; ++c)
          if (lane < 32) red[w * NC + c * 32 + lane] = dot[c];
      }
      __syncthreads();
      if (real && w < NWS) {
        float sacc = auxs[md.bias_off[md.L - 1]];
#pragma unroll
        for (int g = 0; g < 8; ++g) sacc += red[g * NC + tid];
        pend_s = sacc;
        pend_flag = okf[par * NC + tid];
        col_n += (t * NC + tid < ncands ? 1u : 0u) + (pend_flag != 0 ? 0x10000u : 0u);
      }
      // no barrier here: the next tile's first layer reads the input buffer and the bias
      // only; its activations are written behind this barrier, the partial dots and the
      // flags of the other parity behind the next tile's first one
    }
    if (w < NWS) scan_pending();

    if (w < NWS) {
      wave_min(col_v, col_c);
      if (lane == 0) { sv[w] = col_v; sc[w] = col_c; }
      if (stat && col_n) {
        atomicAdd(&sn[0], col_n & 0xffffu);
        atomicAdd(&sn[1], col_n >> 16);
      }
    }
    __syncthreads();
    if (stat && tid == 0 && sn[0]) {
      atomicAdd(&stat[0], (unsigned long long)sn[0]);
      atomicAdd(&stat[1], (unsigned long long)sn[1]);
    }
    float run_v = sv[0];
    int32_t run_c = sc[0];
    if (tid == 0)
      for (int k = 1; k < NWS; ++k) take_min(run_v, run_c, sv[k], sc[k]);
    if (team > 1) {
      // fixed team: every member publishes its minimum, meets the others and reduces all minima.
      // pool: a helper publishes, reports its arrival and is done with the layer; the owner
      // waits for the helpers it sent for and reduces their minima and its own
      const size_t slot0 = ((size_t)(stage & 1) * nprob + unit) * wa.tstride;
      const bool pool = wa.helpers != 0;
      if (tid == 0) {
        if (!pool || helping) {
          wa.team_val[slot0 + member] = run_v;
          wa.team_idx[slot0 + member] = run_c;
          __threadfence();
          atomicAdd(&wa.team_count[unit], 1u);
        }
        if (!pool || !helping) {
          const unsigned int target = pool ? owner_target : (unsigned int)team * (unsigned int)(stage - wa.first + 1);
          unsigned int spins = 0;
          while (__hip_atomic_load(&wa.team_count[unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins > wa.wait_rounds) { team_failed = 1; wa.team_err[0] = 1; break; }
            __builtin_amdgcn_s_sleep(2);
          }
          __threadfence();
        }
      }
      __syncthreads();
      if (team_failed) return;  // a member never arrived: give up instead of waiting for ever
      if (pool && helping) continue;
      if (tid < 64) {
        float v = __builtin_inff();
        int32_t c = -1;
        for (int m = tid; m < team; m += 64) {
          if (pool && m == 0) {  // (thread 0: the owner's own minimum is not published)
            take_min(v, c, run_v, run_c);
            continue;
          }
          const float mv = __hip_atomic_load(&wa.team_val[slot0 + m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const int32_t mc = __hip_atomic_load(&wa.team_idx[slot0 + m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          take_min(v, c, mv, mc);
        }
        wave_min(v, c);
        run_v = v;
        run_c = c;
      }
    } else if (helping) {
      continue;  // (a helper is never sent a layer alone)
    }
    // s_i := the winner; the tables it updates are read back by this same workgroup
    // when it builds the next stage's context
    if (tid == 0)
      commit_winner_call(wa.t.states, wa.t.cf, wa.t.prefix, wa.t.cids, wa.t.vals, wa.t.alive, wa.t.S, pk.d, pk.sp, tabs, unit,
                         stage, run_c, run_v, (uint32_t)M);
    __threadfence();
    __syncthreads();
    // what comes next: an owner goes on to the next layer, then to its next problem; a helper
    // goes back to waiting for an announcement
    if (!helping && ++stage > wa.last) {
      if (wa.helpers && tid == 0) atomicAdd(&wa.pool[2], 1u);
      stage = wa.first;
      unit += (int)gridDim.x / wa.team;
      owner_target = 0u;
    }
  }
}

__global__ __launch_bounds__(256) void k_zero_u32(unsigned int *p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

// Kernel and dynamic LDS bytes of a whole-schedule launch for the context's model.
typedef void (*whole_kernel)(vf_fast_dev, int, int64_t, int, unsigned long long *, NoiseArgs, WholeArgs);
static whole_kernel whole_launch_shape(const vf_ctx *c, vf_fast_dev *fd, int *ks, size_t *smem) {
  int NC = 0;
  vfk_fast_dev(c, true, fd, ks, &NC);
  const size_t aux_words = fd->wl_off + (size_t)(fd->naux - (int)fd->wl_off + 1) / 2;  // output vector: two to a word
  *smem = (size_t)NC * *ks * 2 + (size_t)NC * VF_XIN_STRIDE * 2 + (size_t)8 * NC * 4 + (size_t)2 * NC * 4 + aux_words * 4;
  if (fd->L == 2) return NC == 64 ? k_whole<64, 4, 2, true> : k_whole<128, 2, 4, true>;
  return NC == 64 ? k_whole<64, 4, 2, false> : k_whole<128, 2, 4, false>;
}

// Workgroups per problem for a whole-schedule launch, 0 = use the per-layer launches
// (also when the model's tile does not fit the LDS of a compute unit next to its input
// buffer, e.g. three hidden layers of 512 with all their biases).
// 1 with more problems than half the compute units: every workgroup owns ceil(B / units)
// problems from the first layer to the last and helps the others when it is done (measured
// per step against the per-layer launches: 140 problems 3.6 instead of 5.1 ms, 160: 4.0
// instead of 5.6, 300: 7.0 instead of 8.5); with fewer problems a fixed team per problem, as
// large as the compute units and the tiles of a decision allow, at most 16 (128 problems x
// 2: 3.1 instead of 4.9 ms, 64 x 4: 2.1 instead of 3.4, 32 x 8: 1.7 instead of 2.2; helpers
// instead of fixed teams are slower there: 64 problems 2.9 ms); below 24 problems the
// meetings cost what the launches did.
int vfk_whole_team(const vf_ctx *c) {
  if (!vfk_can_fuse_step(c)) return 0;
  {
    vf_fast_dev fd;
    int ks = 0, lds_max = 0;
    size_t smem = 0;
    const whole_kernel kern = whole_launch_shape(c, &fd, &ks, &smem);
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, (const void *)kern) != hipSuccess) { (void)hipGetLastError(); return 0; }
    (void)hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, c->device);
    if (fd.k0 != VF_K0_OWN || !fd.w_full || fd.L > 3 || smem + attr.sharedSizeBytes > (size_t)lds_max) return 0;
    // The workgroups of this launch wait for each other, so all of them have to be resident at
    // once: the grid is one workgroup per compute unit, and the runtime must say that a compute
    // unit can hold one with this much LDS and these registers (asked once per kernel shape).
    if (c->occ_kern != (const void *)kern || c->occ_smem != smem) {
      int nb = 0;
      if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess ||
          hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void *)kern, 512, smem) != hipSuccess) {
        (void)hipGetLastError();
        nb = 0;
      }
      c->occ_kern = (const void *)kern;
      c->occ_smem = smem;
      c->occ_blocks = nb;
    }
    if (c->occ_blocks < 1) return 0;
  }
  int ncu = 256;
  (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device);
  // (a mailbox names a problem in 23 bits, a layer's tiles are counted in 16)
  if (c->B >= (1 << 23) || (c->M + 63) / 64 > 65535) return 0;
  if (c->B > ncu / 2) return 1;
  if (c->B < 24) return 0;  // a handful of problems: the per-layer launches are faster (16: 1.3 against 1.6 ms)
  int maxw = 0;
  for (int l = 0; l < c->model.n_layers; ++l) if (c->model.dims[l] > maxw) maxw = c->model.dims[l];
  const int NC = maxw > 512 ? 64 : 128;
  const int nparts = (int)((c->M + NC - 1) / NC);
  int team = ncu / c->B;
  if (team > nparts) team = nparts;
  if (team > 16) team = 16;
  // Fixed teams that leave a fifth of the compute units without work, on decisions long enough
  // for helpers to pay (100 rollouts of the 100-stage pipeline, 16384 ids: teams of two use 200
  // of 256 units, 26.9 ms; owners with the other 156 as helpers 25.2 ms; with 4096 ids per
  // decision the teams stay ahead, 2.45 against 2.6 ms)
  if (team >= 2 && (ncu - c->B * team) * 5 >= ncu && nparts >= 64) return 1;
  return team >= 2 ? team : 0;
}

// Algorithm 1 over stages first..last for every problem of the batch, one launch.
int vfk_greedy_whole(vf_ctx *c, int first, int last) {
  const int team = vfk_whole_team(c);
  if (team < 1) return VF_ESTATE;
  const size_t want = (size_t)c->B * c->Mpad;
  if (want > c->wlist_elems) {
    if (c->d_wlist) { VF_HIP(c, hipStreamSynchronize(c->stream)); (void)hipFree(c->d_wlist); c->d_wlist = nullptr; }
    c->wlist_elems = 0;
    if (hipMalloc((void **)&c->d_wlist, want * 4) != hipSuccess) { (void)hipGetLastError(); return VF_ENOMEM; }
    c->wlist_elems = want;
  }
  // meetings: [arrivals B][err 1][pool counters 3][pool queue][mailboxes, 8 bytes per compute unit]
  // [values 2*B*T][ids 2*B*T][published layers B*VF_PUB_WORDS], T slots per problem; everything
  // before the values starts at zero
  int ncu = 256;
  (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device);
  if (ncu >= VF_POOL_SLOTS) return VF_ESTATE;
  const int tstride = team > 1 ? team : 1 + VF_MAX_HELPERS;
  const size_t off_pool = (size_t)c->B + 1, off_q = off_pool + 3;
  const size_t off_mail = (off_q + VF_POOL_SLOTS + 1) & ~(size_t)1;  // 8-byte aligned
  const size_t nzero = off_mail + (size_t)2 * ncu;
  {
    const size_t twant = nzero + (size_t)4 * c->B * tstride + (team == 1 ? (size_t)c->B * VF_PUB_WORDS : 0);
    if (twant > c->team_elems) {
      if (c->d_team) { VF_HIP(c, hipStreamSynchronize(c->stream)); (void)hipFree(c->d_team); c->d_team = nullptr; }
      c->team_elems = 0;
      if (hipMalloc((void **)&c->d_team, twant * 4) != hipSuccess) { (void)hipGetLastError(); return VF_ENOMEM; }
      c->team_elems = twant;
    }
    hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)((nzero + 255) / 256)), dim3(256), 0, c->stream, c->d_team, nzero);
    VF_HIP(c, hipGetLastError());
    if (!c->h_team_err) {
      VF_HIP(c, hipHostMalloc((void **)&c->h_team_err, sizeof(int32_t), hipHostMallocDefault));
      *c->h_team_err = 0;
    }
  }

  vf_fast_dev fd;
  int ks = 0;
  size_t smem = 0;
  const whole_kernel kern = whole_launch_shape(c, &fd, &ks, &smem);
  NoiseArgs na;
  na.eps = c->noise_eps;
  na.k0 = (uint32_t)c->noise_seed; na.k1 = (uint32_t)(c->noise_seed >> 32);
  na.stage = first; na.first_rollout = c->noise_first;
  WholeArgs wa;
  wa.t = tables_of(c);
  wa.first = first; wa.last = last;
  wa.list = reinterpret_cast<uint32_t *>(c->d_wlist); wa.Mpad = c->Mpad;
  wa.team = team;
  wa.helpers = team == 1;
  wa.tstride = tstride;
  wa.team_count = c->d_team;
  wa.team_err = reinterpret_cast<int32_t *>(c->d_team) + c->B;
  wa.wait_rounds = c->wait_rounds;
  wa.pool = c->d_team + off_pool;
  wa.pool_q = c->d_team + off_q;
  wa.mailbox = reinterpret_cast<unsigned long long *>(c->d_team + off_mail);
  wa.team_val = reinterpret_cast<float *>(c->d_team) + nzero;
  wa.team_idx = reinterpret_cast<int32_t *>(c->d_team) + nzero + (size_t)2 * c->B * tstride;
  wa.pub = c->d_team + nzero + (size_t)4 * c->B * tstride;
  // persistent: at most one workgroup per compute unit; with helpers exactly one, so that
  // compute units without a problem of their own help from the start
  const dim3 grid = team > 1 ? dim3((unsigned)(c->B * team)) : dim3((unsigned)ncu);
  {
    vf_prof_scope prof(c, VF_PROF_SCORE);
    VF_HIP(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(kern, grid, dim3(512), smem, c->stream, fd, ks, c->M, c->B,
                       c->profiling ? c->d_stat : (unsigned long long *)nullptr, na, wa);
    VF_HIP(c, hipGetLastError());
  }
  c->dec_stage = -1;
  // the flag of a wait that ran out, and an event behind its copy: whoever looks at the flag
  // waits for (or polls) the event first
  VF_HIP(c, hipMemcpyAsync(c->h_team_err, reinterpret_cast<int32_t *>(c->d_team) + c->B, sizeof(int32_t),
                             hipMemcpyDeviceToHost, c->stream));
  if (!c->ev_whole) VF_HIP(c, hipEventCreateWithFlags(&c->ev_whole, hipEventDisableTiming));
  VF_HIP(c, hipEventRecord(c->ev_whole, c->stream));
  c->whole_pending = true;
  c->whole_first = first;
  c->whole_last = last;
  c->whole_epoch = c->state_epoch;
  return VF_OK;
}
