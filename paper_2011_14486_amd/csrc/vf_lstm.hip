// The recurrent value network of Sec. 3.2 wired to the search (gfx950).
//
// V reads a state as a sequence with one timestep per stage of the pipeline, in
// scheduling order: a stage that is scheduled in the state gives its 64 core features,
// a stage that is not gives its intrinsic block and zeros; every timestep's hidden
// state goes through the linear head and the predictions are summed.  For the
// candidates of decision i all timesteps before i are the same, so the recurrence over
// the committed prefix is kept per problem (cell state, the fed-back h folded into the
// gate pre-activations of the next step, the head's sum so far) and advanced by one
// step at every commit.  A candidate then costs one cell step on its own features plus
// one step per stage still unscheduled; for those the input part of the gates does not
// depend on the candidate either and comes from a per-problem table.
#include "vf_internal.h"

namespace {

#include "vf_sched_dev.h"
#include "vf_score_dev.h"

// fp32 blob of the model: W_ih[4H][64], W_hh[4H][H], b_ih[4H], b_hh[4H], w_head[H], b_head
struct SeqWeights {
  const float *Wih, *Whh, *bih, *bhh, *wh, *bh;
  int H;
};

__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// G[b][t][r] = b_ih[r] + b_hh[r] + sum_{k<16} W_ih[r][k] x_k, x = the normalised intrinsic
// block of stage t: the input part of the gates of a stage that is not scheduled yet.
__global__ __launch_bounds__(256) void k_seq_tables(const int32_t *intr, SeqWeights sw, size_t n_bt, float *G) {
  const int H4 = 4 * sw.H;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_bt * (size_t)H4) return;
  const size_t bt = i / H4;
  const int r = (int)(i % H4);
  float acc = 0.0f;
#pragma unroll
  for (int k = 0; k < 16; ++k)
    acc = fmaf(bf16_val(sw.Wih[(size_t)r * 64 + k]), bf16_val(plog2_dev(intr[bt * 16 + k])), acc);
  G[i] = acc + sw.bih[r] + sw.bhh[r];
}

// the recurrence before the first stage: h = c = 0, so the gates start from the biases
__global__ __launch_bounds__(256) void k_seq_reset(SeqWeights sw, int B, float *hfb, float *cpre, float *P,
                                                   float *hsum) {
  const int H = sw.H;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < (size_t)B * H) { hfb[i] = 0.0f; cpre[i] = 0.0f; }
  if (i < (size_t)B * 4 * H) P[i] = sw.bih[i % (4 * H)] + sw.bhh[i % (4 * H)];
  if (i < (size_t)B) hsum[i] = 0.0f;
}

// One cell step per problem on the vector committed for `stage`; then the part of the
// next step's gates that comes from the new h.  A problem whose schedule has ended
// keeps its state (it has no candidates any more).  With sel_idx (beam search) slot b
// of the dst set continues the recurrence of its parent slot sel_idx[b] / Mpad of the
// src set; slots past the sel_n[0] survivors are dead and left alone.
struct SeqState {
  float *hfb, *cpre, *P, *hsum;  // [B][H] (bf16 values), [B][H], [B][4H], [B]
};

constexpr int SEQ_PB = 4;  // problems per workgroup of k_seq_advance: they share the weight reads

// [W_ih | W_hh] transposed and rounded: WT[k][r], k over the 64 inputs then the H hidden
// units, r over the 4H gate rows, so that thread r of a block reads its row coalesced.
__global__ __launch_bounds__(256) void k_pack_seqT(SeqWeights sw, float *WT) {
  const int H = sw.H, H4 = 4 * H;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)(64 + H) * H4) return;
  const int k = (int)(i / H4), r = (int)(i % H4);
  WT[i] = bf16_val(k < 64 ? sw.Wih[(size_t)r * 64 + k] : sw.Whh[(size_t)r * H + (k - 64)]);
}

__global__ __launch_bounds__(1024) void k_seq_advance(Tables t, int stage, SeqWeights sw, const float *WT, SeqState src,
                                                      SeqState dst, const int32_t *sel_idx, const int32_t *sel_n,
                                                      int64_t Mpad, int B) {
  __shared__ float x[SEQ_PB][64], z[SEQ_PB][1024], hn[SEQ_PB][256], hraw[SEQ_PB][256];
  __shared__ int from_s[SEQ_PB], mode_s[SEQ_PB];  // 0: leave alone, 1: carry the state over, 2: one cell step
  const int tid = threadIdx.x, lane = tid & 63;
  const int H = sw.H, H4 = 4 * H, S = t.S;
  const int b0 = blockIdx.x * SEQ_PB;
  if (tid < SEQ_PB) {
    const int b = b0 + tid;
    int mode = 0, from = b;
    if (b < B) {
      const bool survivor = !sel_idx || b < sel_n[0];  // beam search: slots past the survivors are dead
      if (survivor) {
        if (sel_idx) from = (int)((int64_t)sel_idx[b] / Mpad);
        const bool live = t.cids[(size_t)b * S + stage] >= 0;
        mode = live ? 2 : (src.cpre != dst.cpre ? 1 : 0);
      }
    }
    from_s[tid] = from;
    mode_s[tid] = mode;
  }
  __syncthreads();
  for (int i = tid; i < SEQ_PB * 64; i += 1024) {
    const int pb = i / 64, k = i % 64;
    x[pb][k] = mode_s[pb] == 2 ? bf16_val(plog2_dev(t.cf[((size_t)(b0 + pb) * S + stage) * 64 + k])) : 0.0f;
  }
  __syncthreads();
  // gate pre-activations: thread r owns row r for the block's problems
  if (tid < H4) {
    float acc[SEQ_PB];
#pragma unroll
    for (int pb = 0; pb < SEQ_PB; ++pb) acc[pb] = 0.0f;
#pragma unroll 16
    for (int k = 0; k < 64; ++k) {
      const float wv = WT[(size_t)k * H4 + tid];
#pragma unroll
      for (int pb = 0; pb < SEQ_PB; ++pb) acc[pb] = fmaf(wv, x[pb][k], acc[pb]);
    }
#pragma unroll
    for (int pb = 0; pb < SEQ_PB; ++pb)
      if (mode_s[pb] == 2) z[pb][tid] = src.P[(size_t)from_s[pb] * H4 + tid] + acc[pb];
  }
  __syncthreads();
  for (int i = tid; i < SEQ_PB * H; i += 1024) {
    const int pb = i / H, u = i % H, b = b0 + pb, from = from_s[pb];
    if (mode_s[pb] == 2) {
      float cn = src.cpre[(size_t)from * H + u];
      const float h = lstm_cell(z[pb][u], z[pb][H + u], z[pb][2 * H + u], z[pb][3 * H + u], cn);
      dst.cpre[(size_t)b * H + u] = cn;
      hraw[pb][u] = h;
      hn[pb][u] = bf16_val(h);
      dst.hfb[(size_t)b * H + u] = hn[pb][u];
    } else if (mode_s[pb] == 1) {
      dst.cpre[(size_t)b * H + u] = src.cpre[(size_t)from * H + u];
      dst.hfb[(size_t)b * H + u] = src.hfb[(size_t)from * H + u];
    }
  }
  __syncthreads();
  // the head's prediction for this timestep: one wave per problem, fixed order
  if (tid < SEQ_PB * 64) {
    const int pb = tid / 64;
    if (mode_s[pb] == 2) {
      float v = 0.0f;
      for (int u = lane; u < H; u += 64) v = fmaf(bf16_val(sw.wh[u]), hraw[pb][u], v);
      v = wave_sum(v);
      if (lane == 0) dst.hsum[b0 + pb] = src.hsum[from_s[pb]] + v + sw.bh[0];
    } else if (mode_s[pb] == 1 && lane == 0) {
      dst.hsum[b0 + pb] = src.hsum[from_s[pb]];
    }
  }
  // the h part of the next step's gates
  if (tid < H4) {
    float acc[SEQ_PB];
#pragma unroll
    for (int pb = 0; pb < SEQ_PB; ++pb) acc[pb] = 0.0f;
#pragma unroll 16
    for (int k = 0; k < H; ++k) {
      const float wv = WT[(size_t)(64 + k) * H4 + tid];
#pragma unroll
      for (int pb = 0; pb < SEQ_PB; ++pb) acc[pb] = fmaf(wv, hn[pb][k], acc[pb]);
    }
    const float bias = sw.bih[tid] + sw.bhh[tid];
#pragma unroll
    for (int pb = 0; pb < SEQ_PB; ++pb) {
      if (mode_s[pb] == 2) dst.P[(size_t)(b0 + pb) * H4 + tid] = bias + acc[pb];
      else if (mode_s[pb] == 1) dst.P[(size_t)(b0 + pb) * H4 + tid] = src.P[(size_t)from_s[pb] * H4 + tid];
    }
  }
}

// The valid candidates of decision (problem b, stage), in ascending id order:
// list[b][0..count[b]).  The recurrent network costs one cell step per remaining stage and
// candidate, so the scoring kernel works on this dense list instead of the id range, where
// valid and invalid ids are interleaved.  Also fills the masked score array (nullable)
// with +inf: the scorer then only writes the candidates' entries.
__global__ __launch_bounds__(1024) void k_seq_compact(const uint32_t *decpack, uint32_t M, int64_t Mpad, int32_t *list,
                                                      int32_t *count, float *scores) {
  __shared__ DecPack pk;
  __shared__ int wsum[16];
  __shared__ int base;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid < VF_DECPACK_DWORDS) reinterpret_cast<uint32_t *>(&pk)[tid] = decpack[(size_t)b * VF_DECPACK_DWORDS + tid];
  if (tid == 0) base = 0;
  __syncthreads();
  for (uint32_t c0 = 0; c0 < (uint32_t)Mpad; c0 += 1024u) {
    const uint32_t cid = c0 + tid;
    bool ok = false;
    if (cid < M && !range_closed(pk.d, pk.sp, c0, c0 + 1024u < M ? c0 + 1024u : M)) {
      uint32_t dec;
      ok = eval_candidate<false>(pk.d, pk.sp, cid, dec, nullptr);
    }
    if (scores && cid < (uint32_t)Mpad) scores[(size_t)b * Mpad + cid] = __builtin_inff();
    const unsigned long long m = __ballot(ok);
    if (lane == 0) wsum[w] = __popcll(m);
    __syncthreads();
    int off = base;
    for (int k = 0; k < w; ++k) off += wsum[k];
    if (ok) list[(size_t)b * Mpad + off + __popcll(m & ((1ull << lane) - 1ull))] = (int32_t)cid;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int k = 0; k < 16; ++k) tot += wsum[k];
      base += tot;
    }
    __syncthreads();
  }
  if (tid == 0) count[b] = base;
}

struct SeqDev {
  int H, S;
  const uint16_t *w_pack;  // [unit tile][k step][gate][lane][8]; 4 k-steps of x, then H/16 of h
  const float *aux;        // b_ih + b_hh [4H], head vector [H] (bf16 values), head bias
  const float *G;          // [B][S][4H]
  const float *P;          // [B][4H]
  const float *cpre;       // [B][H]
  const float *hsum;       // [B]
  const uint32_t *decpack; // [B][VF_DECPACK_DWORDS]
  const int32_t *list;     // [B][Mpad] valid candidate ids of the decision, ascending
  const int32_t *count;    // [B]
  int64_t Mpad;
  unsigned long long *stat;
};

// Workgroup = NC consecutive entries of the valid-candidate list of decision `stage` of
// problem blockIdx.y: featurize them, one cell step on their features from the problem's prefix state, one
// step per later stage, the head's sum, the tile's first minimum.  Wave w owns hidden
// units 32w..32w+31 (their four gate row tiles); c lives in registers, h goes through
// LDS as bf16, double-buffered; the weight fragments of a step are one contiguous stream
// per wave, kept PD k-steps ahead in a register ring that wraps at the end of the step;
// the per-step gate biases of the problem are staged through LDS one step ahead.
template <int NC, int PD>
__global__ __launch_bounds__(512) void k_seq_step(SeqDev md, int stage, int64_t M, float *scores, int64_t ld_scores,
                                                  float *pval, int32_t *pidx, NoiseArgs na) {
  constexpr int CT = NC / 32;
  constexpr int XLD = 72;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int H = md.H, S = md.S, H4 = 4 * H, hld = H + 8;
  uint16_t *xs = reinterpret_cast<uint16_t *>(smem);                    // [NC][XLD]
  uint16_t *hs = xs + (size_t)NC * XLD;                                 // [2][NC][hld]
  float *gls = reinterpret_cast<float *>(hs + (size_t)2 * NC * hld);    // [2][4H]
  float *red = gls + 2 * H4;                                            // [8][NC]
  float *whs = red + 8 * NC;                                            // [H]
  int32_t *okf = reinterpret_cast<int32_t *>(whs + H);                  // [NC]
  int32_t *cids = okf + NC;                                             // [NC] candidate id of each column
  __shared__ DecPack pk;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y, nparts = gridDim.x;
  const int64_t n0 = (int64_t)blockIdx.x * NC;
  const size_t slot = (size_t)b * nparts + blockIdx.x;

  if (tid < VF_DECPACK_DWORDS)
    reinterpret_cast<uint32_t *>(&pk)[tid] = md.decpack[(size_t)b * VF_DECPACK_DWORDS + tid];
  __syncthreads();

  const int nvalid = md.count[b];
  if (n0 >= nvalid) {
    // past the end of the list: nothing for the network to do
    if (tid == 0) {
      pval[slot] = __builtin_inff();
      pidx[slot] = -1;
    }
    return;
  }
  // four threads per candidate, each producing 16 of the 64 core rows
  if (tid < NC) cids[tid] = (n0 + tid) < nvalid ? md.list[(size_t)b * md.Mpad + n0 + tid] : -1;
  if (tid < 4 * NC) {
    const int n = tid % NC, part = tid / NC;
    const bool inb = (n0 + n) < nvalid;
    const uint32_t cid = inb ? (uint32_t)md.list[(size_t)b * md.Mpad + n0 + n] : 0u;
    int32_t core[64];
    uint32_t dec;
    // the parts a thread does not store are dead code in its copy of the evaluation
    auto put = [&](const int32_t *v, int row0) {
      uint4 q0, q1;
      q0.x = pack_bf16(plog2_dev(v[0]), plog2_dev(v[1]));
      q0.y = pack_bf16(plog2_dev(v[2]), plog2_dev(v[3]));
      q0.z = pack_bf16(plog2_dev(v[4]), plog2_dev(v[5]));
      q0.w = pack_bf16(plog2_dev(v[6]), plog2_dev(v[7]));
      q1.x = pack_bf16(plog2_dev(v[8]), plog2_dev(v[9]));
      q1.y = pack_bf16(plog2_dev(v[10]), plog2_dev(v[11]));
      q1.z = pack_bf16(plog2_dev(v[12]), plog2_dev(v[13]));
      q1.w = pack_bf16(plog2_dev(v[14]), plog2_dev(v[15]));
      if (!inb) q0 = q1 = make_uint4(0u, 0u, 0u, 0u);
      uint4 *dst = reinterpret_cast<uint4 *>(xs + (size_t)n * XLD + row0);
      dst[0] = q0;
      dst[1] = q1;
    };
    if (part == 0) {
      // evaluated for padding columns too: core must be defined before put reads it
      const bool okc = eval_candidate<true>(pk.d, pk.sp, cid, dec, core);
      okf[n] = inb && okc;
      put(core, 0);
    } else if (part == 1) {
      eval_candidate<true>(pk.d, pk.sp, cid, dec, core);
      put(core + 16, 16);
    } else if (part == 2) {
      eval_candidate<true>(pk.d, pk.sp, cid, dec, core);
      put(core + 32, 32);
    } else {
      eval_candidate<true>(pk.d, pk.sp, cid, dec, core);
      put(core + 48, 48);
    }
  }

  const bool active = w < H / 32;
  const int wu = active ? w : 0;  // idle waves shadow tile 0 but never store
  const int ksh = H / 16, ksteps = 4 + ksh;
  // the wave's weight stream (4 k-steps of x part, then the h part): base in scalar registers,
  // 16 bytes per lane, fragment i at byte 1024 i
  const __amdgpu_buffer_rsrc_t ws = stream_rsrc(reinterpret_cast<const uint4 *>(md.w_pack) + (size_t)wu * ksteps * 4 * 64);
  const int voff = 16 * lane;
  int wstep = PD;  // the k-step of the stream that refills the next slot
  uint4 ring[PD][4];
#pragma unroll
  for (int j = 0; j < PD; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) ring[j][g] = stream_load(ws, voff, j * 4 + g);

  for (int i = tid; i < H4; i += 512) gls[i] = md.P[(size_t)b * H4 + i];
  for (int i = tid; i < H; i += 512) whs[i] = md.aux[H4 + i];
  floatx16 cst[CT];
  float vsum[CT];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float4 cv = *reinterpret_cast<const float4 *>(md.cpre + (size_t)b * H + wu * 32 + 4 * (lane >> 5) + 8 * q);
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      cst[c][4 * q + 0] = cv.x; cst[c][4 * q + 1] = cv.y;
      cst[c][4 * q + 2] = cv.z; cst[c][4 * q + 3] = cv.w;
    }
  }
#pragma unroll
  for (int c = 0; c < CT; ++c) vsum[c] = 0.0f;
  __syncthreads();

  const int rowoff = (lane & 31), koff = 8 * (lane >> 5);
  for (int t = stage; t < S; ++t) {
    const int k = t - stage;
    // the next step's biases, fetched now, parked in LDS after this step's contraction
    const bool fetch_g = (t + 1 < S) && tid < H;
    float4 gnext = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (fetch_g) gnext = reinterpret_cast<const float4 *>(md.G + ((size_t)b * S + t + 1) * H4)[tid];

    // the step's gate biases (staged in LDS one step ahead) are the addends of the first k-step:
    // gate by gate, so that one bias vector is in registers at a time
    const float *bias = gls + (size_t)(k & 1) * H4;
    floatx16 acc[4][CT];

    const uint16_t *src = (k == 0) ? xs : hs + (size_t)(k & 1) * NC * hld;
    const int ld = (k == 0) ? XLD : hld;
    const int nsteps = (k == 0) ? 4 : ksh;
    {
      const uint16_t *brow = src + (size_t)rowoff * ld + koff;
      uint4 bcur[CT];
#pragma unroll
      for (int c = 0; c < CT; ++c) bcur[c] = *reinterpret_cast<const uint4 *>(brow + (size_t)c * 32 * ld);
      auto round = [&](int s0, auto startc) __attribute__((always_inline)) {
        constexpr bool starts = decltype(startc)::value;
        if (s0 + PD >= nsteps) wstep = 4;  // the next step's first fragments (always an h step)
#pragma unroll
        for (int j = 0; j < PD; ++j) {
          if constexpr (starts) {
            if (j == 0) {
              int boff = wu * 32 + 4 * (lane >> 5);
              asm volatile("" : "+v"(boff));  // (read afresh every step, not kept across them)
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                floatx16 bg;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                  const float4 bv = *reinterpret_cast<const float4 *>(bias + g * H + boff + 8 * q);
                  bg[4 * q + 0] = bv.x; bg[4 * q + 1] = bv.y; bg[4 * q + 2] = bv.z; bg[4 * q + 3] = bv.w;
                }
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                  acc[g][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                      __builtin_bit_cast(bf16x8, ring[0][g]), __builtin_bit_cast(bf16x8, bcur[c]), bg, 0, 0, 0);
                  if (g == 3) bcur[c] = *reinterpret_cast<const uint4 *>(brow + (size_t)c * 32 * ld + 16);
                }
                ring[0][g] = stream_load(ws, voff, wstep * 4 + g);
              }
              continue;
            }
          }
          // column by column; every operand register is refilled in place behind the last product
          // that reads it: a column's activation fragment with the next k-step's (one k-step
          // past the end stays inside the row's padding or the next row), a weight fragment
          // with the one PD k-steps ahead
#pragma unroll
          for (int i = 0; i < 4 * CT; ++i) {
            const int c = i / 4, g = i % 4;
            acc[g][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, ring[j][g]), __builtin_bit_cast(bf16x8, bcur[c]), acc[g][c], 0, 0, 0);
            if (g == 3) bcur[c] = *reinterpret_cast<const uint4 *>(brow + (size_t)c * 32 * ld + (s0 + j + 1) * 16);
            if (c == CT - 1) ring[j][g] = stream_load(ws, voff, (wstep + j) * 4 + g);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        wstep += PD;
      };
      round(0, vf_tag<true>{});
      for (int s0 = PD; s0 < nsteps; s0 += PD) round(s0, vf_tag<false>{});
    }
    if (fetch_g) reinterpret_cast<float4 *>(gls + (size_t)((k + 1) & 1) * H4)[tid] = gnext;

    uint16_t *hout = hs + (size_t)((k + 1) & 1) * NC * hld;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int u0 = wu * 32 + 4 * (lane >> 5) + 8 * q;
      const float4 whv = *reinterpret_cast<const float4 *>(whs + u0);
      const float whq[4] = {whv.x, whv.y, whv.z, whv.w};
#pragma unroll
      for (int c = 0; c < CT; ++c) {
        float hv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = 4 * q + e;
          float cn = cst[c][j];
          hv[e] = lstm_cell(acc[0][c][j], acc[1][c][j], acc[2][c][j], acc[3][c][j], cn);
          cst[c][j] = cn;
          vsum[c] = fmaf(whq[e], hv[e], vsum[c]);
        }
        if (active) {
          uint2 pkd;
          pkd.x = pack_bf16(hv[0], hv[1]);
          pkd.y = pack_bf16(hv[2], hv[3]);
          *reinterpret_cast<uint2 *>(hout + (size_t)(c * 32 + (lane & 31)) * hld + u0) = pkd;
        }
      }
    }
    __syncthreads();  // h_t and the next step's biases are in place
  }

#pragma unroll
  for (int c = 0; c < CT; ++c) {
    const float v = vsum[c] + __shfl_xor(vsum[c], 32);
    if (lane < 32) red[w * NC + c * 32 + lane] = active ? v : 0.0f;
  }
  __syncthreads();
  if (tid < NC) {
    float s = md.hsum[b] + (float)(S - stage) * md.aux[H4 + H];
#pragma unroll
    for (int g = 0; g < 8; ++g) s += red[g * NC + tid];
    const bool ok = okf[tid] != 0;
    const int32_t cid = cids[tid];
    if (scores && ok) scores[(size_t)b * ld_scores + cid] = s;
    if (na.eps != 0.0f) s = add_noise(na, s, b, cid);
    float v = __builtin_inff();
    int32_t c = -1;
    if (ok && s < v) { v = s; c = cid; }
    wave_min(v, c);
    if (md.stat) {
      const int nok = __popcll(__ballot(ok));
      if (lane == 0) {
        atomicAdd(&md.stat[0], (unsigned long long)nok);
        atomicAdd(&md.stat[1], (unsigned long long)nok);
      }
    }
    if (tid == 0) {
      pval[slot] = v;
      pidx[slot] = c;
    }
  }
}

SeqWeights weights_of(const vf_ctx *c) {
  const int H = c->model.dims[1];
  SeqWeights sw;
  sw.H = H;
  sw.Wih = c->pm.w_f32;
  sw.Whh = sw.Wih + (size_t)4 * H * 64;
  sw.bih = sw.Whh + (size_t)4 * H * H;
  sw.bhh = sw.bih + 4 * H;
  sw.wh = sw.bhh + 4 * H;
  sw.bh = sw.wh + H;
  return sw;
}

SeqState state_of(const vf_ctx *c, int set) {
  SeqState s;
  s.hfb = c->d_seq_h[set]; s.cpre = c->d_seq_c[set]; s.P = c->d_seq_P[set]; s.hsum = c->d_seq_hs[set];
  return s;
}

}  // namespace

bool vfk_seq_model(const vf_ctx *c) {
  return c->has_model && c->model.kind == VF_LSTM && c->model.dtype == VF_BF16 && c->model.dims[0] == 64 &&
         c->pm.w_f32 != nullptr;
}

void vfk_seq_free(vf_ctx *c) {
  void *ps[] = {c->d_seq_G, c->d_seq_h[0], c->d_seq_h[1], c->d_seq_c[0], c->d_seq_c[1],
                c->d_seq_P[0], c->d_seq_P[1], c->d_seq_hs[0], c->d_seq_hs[1], c->d_seq_list, c->d_seq_count};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  c->d_seq_G = nullptr;
  c->d_seq_list = nullptr;
  c->d_seq_count = nullptr;
  for (int k = 0; k < 2; ++k) c->d_seq_h[k] = c->d_seq_c[k] = c->d_seq_P[k] = c->d_seq_hs[k] = nullptr;
  c->seq_stage = -1;
  c->seq_cur = 0;
}

// Tables and prefix state of the recurrence for the context's pipeline, model and
// committed prefix: built on first use, rebuilt after anything but a commit changed them.
int vfk_seq_sync(vf_ctx *c, int stage) {
  const int H = c->model.dims[1], B = c->B, S = c->S;
  const SeqWeights sw = weights_of(c);
  hipStream_t st = c->stream;
  if (!c->d_seq_G) {
    struct { float **p; size_t n; } want[] = {
        {&c->d_seq_G, (size_t)B * S * 4 * H},
        {&c->d_seq_h[0], (size_t)B * H}, {&c->d_seq_h[1], (size_t)B * H},
        {&c->d_seq_c[0], (size_t)B * H}, {&c->d_seq_c[1], (size_t)B * H},
        {&c->d_seq_P[0], (size_t)B * 4 * H}, {&c->d_seq_P[1], (size_t)B * 4 * H},
        {&c->d_seq_hs[0], (size_t)B}, {&c->d_seq_hs[1], (size_t)B}};
    bool ok = true;
    for (auto &wt : want) ok = ok && hipMalloc((void **)wt.p, wt.n * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->d_seq_list, (size_t)B * c->Mpad * 4) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->d_seq_count, (size_t)B * 4) == hipSuccess;
    if (!ok) {
      (void)hipGetLastError();
      vfk_seq_free(c);
      return VF_ENOMEM;
    }
    const size_t n = (size_t)B * S * 4 * H;
    hipLaunchKernelGGL(k_seq_tables, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, c->d_intr, sw,
                       (size_t)B * S, c->d_seq_G);
    VF_HIP(c, hipGetLastError());
    if (!c->pm.w_seqT) {
      const size_t nw = (size_t)(64 + H) * 4 * H;
      if (hipMalloc((void **)&c->pm.w_seqT, nw * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        vfk_seq_free(c);
        return VF_ENOMEM;
      }
      hipLaunchKernelGGL(k_pack_seqT, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, st, sw, c->pm.w_seqT);
      VF_HIP(c, hipGetLastError());
    }
    c->seq_stage = -1;
  }
  if (c->seq_stage == stage) return VF_OK;
  c->seq_cur = 0;
  const size_t n = (size_t)B * 4 * H;
  const SeqState s0 = state_of(c, 0);
  hipLaunchKernelGGL(k_seq_reset, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sw, B, s0.hfb, s0.cpre, s0.P,
                     s0.hsum);
  VF_HIP(c, hipGetLastError());
  for (int t = 0; t < stage; ++t) {
    hipLaunchKernelGGL(k_seq_advance, dim3((unsigned)((B + SEQ_PB - 1) / SEQ_PB)), dim3(1024), 0, st, tables_of(c), t, sw,
                       (const float *)c->pm.w_seqT, s0, s0, (const int32_t *)nullptr, (const int32_t *)nullptr,
                       (int64_t)c->Mpad, B);
    VF_HIP(c, hipGetLastError());
  }
  c->seq_stage = stage;
  return VF_OK;
}

// after the commit of `stage`: one more step of every problem's prefix recurrence
int vfk_seq_advance(vf_ctx *c, int stage) {
  if (c->seq_stage != stage) return VF_OK;  // not in step: rebuilt at the next use
  const SeqState s = state_of(c, c->seq_cur);
  hipLaunchKernelGGL(k_seq_advance, dim3((unsigned)((c->B + SEQ_PB - 1) / SEQ_PB)), dim3(1024), 0, c->stream,
                     tables_of(c), stage, weights_of(c), (const float *)c->pm.w_seqT, s, s, (const int32_t *)nullptr,
                     (const int32_t *)nullptr, (int64_t)c->Mpad, c->B);
  VF_HIP(c, hipGetLastError());
  c->seq_stage = stage + 1;
  return VF_OK;
}

// beam search: slot j of the new layer continues the recurrence of its parent slot
int vfk_seq_advance_beam(vf_ctx *c, int stage) {
  if (c->seq_stage != stage) return VF_OK;
  const SeqState src = state_of(c, c->seq_cur), dst = state_of(c, c->seq_cur ^ 1);
  hipLaunchKernelGGL(k_seq_advance, dim3((unsigned)((c->B + SEQ_PB - 1) / SEQ_PB)), dim3(1024), 0, c->stream,
                     tables_of(c), stage, weights_of(c), (const float *)c->pm.w_seqT, src, dst,
                     (const int32_t *)c->d_sel_idx, (const int32_t *)c->d_sel_n, (int64_t)c->Mpad, c->B);
  VF_HIP(c, hipGetLastError());
  c->seq_cur ^= 1;
  c->seq_stage = stage + 1;
  return VF_OK;
}

// V of every candidate state of decision `stage` of every problem: per-tile minima into
// the partial arrays, optionally the masked scores [B][ld_scores].
int vfk_seq_step(vf_ctx *c, int stage, float *scores, int64_t ld_scores, int noise_stage, int *nparts_out) {
  constexpr int NC = 64;
  int rc = vfk_seq_sync(c, stage);
  if (rc != VF_OK) return rc;
  rc = vfk_prepare(c, stage);
  if (rc != VF_OK) return rc;
  const int H = c->model.dims[1];
  const int nparts = (int)((c->M + NC - 1) / NC);
  rc = vfk_ensure_parts(c, (size_t)nparts * c->B);
  if (rc != VF_OK) return rc;
  const SeqState s = state_of(c, c->seq_cur);
  SeqDev md;
  md.H = H; md.S = c->S; md.w_pack = c->pm.w_pack; md.aux = c->pm.aux;
  md.G = c->d_seq_G; md.P = s.P; md.cpre = s.cpre; md.hsum = s.hsum;
  md.decpack = c->d_decpack;
  md.list = c->d_seq_list; md.count = c->d_seq_count; md.Mpad = c->Mpad;
  md.stat = c->profiling ? c->d_stat : nullptr;
  hipLaunchKernelGGL(k_seq_compact, dim3((unsigned)c->B), dim3(1024), 0, c->stream, c->d_decpack, (uint32_t)c->M,
                     (int64_t)c->Mpad, c->d_seq_list, c->d_seq_count, scores);
  VF_HIP(c, hipGetLastError());
  NoiseArgs na;
  na.eps = noise_stage >= 0 ? c->noise_eps : 0.0f;
  na.k0 = (uint32_t)c->noise_seed; na.k1 = (uint32_t)(c->noise_seed >> 32);
  na.stage = noise_stage; na.first_rollout = c->noise_first;
  const int hld = H + 8;
  const size_t smem = (size_t)NC * 72 * 2 + (size_t)2 * NC * hld * 2 + (size_t)2 * 4 * H * 4 + (size_t)8 * NC * 4 +
                      (size_t)H * 4 + (size_t)2 * NC * 4;
  {
    vf_prof_scope prof(c, VF_PROF_SCORE);
    void (*kern)(SeqDev, int, int64_t, float *, int64_t, float *, int32_t *, NoiseArgs) = k_seq_step<NC, 2>;
    VF_HIP(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(kern, dim3((unsigned)nparts, (unsigned)c->B), dim3(512), smem, c->stream, md, stage, c->M,
                       scores, ld_scores, c->d_pval, c->d_pidx, na);
    VF_HIP(c, hipGetLastError());
  }
  *nparts_out = nparts;
  return VF_OK;
}
