// Value networks V(s) and the argmin scan of Algorithm 1 (gfx950).
//
// Inputs are raw integer features, candidate-contiguous ([feature][candidate]); they
// are normalised on load with a piecewise-linear log2 (Sec. 3.2: the network is fed
// normalised feature values).  Three scorers:
//   - fp32 MLP: plain FMA kernels, one layer per launch (small models);
//   - bf16 MLP: the whole layer chain in one kernel per tile of candidates.  The
//     tile's activations live in LDS as bf16 [candidate][feature]; weights are the
//     MFMA A operand (output feature = row), activations the B operand (candidate =
//     column), so the 32x32 accumulator of a lane holds 4x4 consecutive features of
//     one candidate and goes back to LDS with 8-byte writes.  Weights are repacked
//     once into A-fragment order and stream from L2 straight into registers;
//   - bf16 LSTM (Sec. 3.2): per timestep one [4H] x [F+H] contraction per candidate
//     tile, gates and cell state in fp32 registers, h_t fed back through LDS as
//     bf16, the per-timestep linear prediction accumulated on the fly.
// Every scoring workgroup also reduces its candidates to one (value, id) pair: the
// inner loop "if V(s) < v_i" of Algorithm 1 keeps the first strict minimum, so the
// reduction orders by value, then by id, and NaN never wins.
#include <stdlib.h>

#include <mutex>

#include "vf_internal.h"

// Scratch of vf_score_static (the entry point that allocates nothing): the per-workgroup
// (value, id) minima that the scoring kernel leaves for the group scan, VF_STATIC_PARTS
// floats followed by as many ids.  Every GPU the library runs on holds its own copy at its
// own address until the process ends; in host code the name below is only a handle for
// hipGetSymbolAddress, never a device address.
// (VF_STATIC_PARTS = 65536 pairs = 512 KiB; tiles of 64 candidates: up to 4,194,304 candidates per call)
static __device__ __align__(256) unsigned char scratch[(size_t)VF_STATIC_PARTS * 8];

namespace {

#include "vf_sched_dev.h"

#include "vf_score_dev.h"

// --------------------------------------------------------------- fp32 MLP

// Wt[k][o] = W[o][k] for o < N, zero up to Npad
__global__ __launch_bounds__(256) void k_transpose_f32(const float *W, int K, int N, int Npad, float *Wt) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)K * Npad) return;
  const int k = (int)(i / Npad), o = (int)(i % Npad);
  Wt[i] = o < N ? W[(size_t)o * K + k] : 0.0f;
}

// out[o][n] = act(b[o] + sum_k W[o][k] * in[k][n]); one thread per candidate, 16
// outputs per thread; the weights come transposed (Wt[k][Npad]), so that the 16 a thread needs
// for one k are one uniform 64-byte read, and four rows of the input are fetched at a time;
// every accumulator adds its products in the order k = 0, 1, 2, ...
template <bool FIRST>
__global__ __launch_bounds__(256) void k_mlp_f32_layer(const void *in_, int64_t in_stride, int64_t ld_in,
                                                       const float *__restrict__ Wt, int Npad, const float *bias, float *out,
                                                       int64_t out_stride, int64_t ld_out, int K, int N,
                                                       int64_t M, int relu) {
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int o0 = blockIdx.y * 16;
  const int p = blockIdx.z;
  if (n >= M) return;
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
  const int32_t *xi = (const int32_t *)in_ + (size_t)p * in_stride;
  const float *xf = (const float *)in_ + (size_t)p * in_stride;
#pragma unroll 4
  for (int k = 0; k < K; ++k) {
    float a = FIRST ? plog2_dev(xi[(size_t)k * ld_in + n]) : xf[(size_t)k * ld_in + n];
    const float *wrow = Wt + (size_t)k * Npad + o0;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = fmaf(wrow[j], a, acc[j]);  // (padding: zero weights, never stored)
  }
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if (o0 + j < N) {
      float v = acc[j] + bias[o0 + j];
      if (relu) v = relu_keep_nan(v);
      out[(size_t)p * out_stride + (size_t)(o0 + j) * ld_out + n] = v;
    }
}

// One (value, id) pair per block of VF_PART candidates of each problem.
__global__ __launch_bounds__(VF_PART) void k_argmin_parts(const float *scores, int64_t score_stride,
                                                          const int32_t *valid_row, int64_t valid_stride,
                                                          int64_t M, int nparts, float *pval, int32_t *pidx,
                                                          NoiseArgs na) {
  __shared__ float sv[VF_PART / 64];
  __shared__ int32_t sc[VF_PART / 64];
  const int p = blockIdx.y;
  const int64_t n = (int64_t)blockIdx.x * VF_PART + threadIdx.x;
  float v = __builtin_inff();
  int32_t c = -1;
  if (n < M) {
    float s = scores[(size_t)p * score_stride + n];
    bool ok = valid_row ? valid_row[(size_t)p * valid_stride + n] != 0 : true;
    if (na.eps != 0.0f) s = add_noise(na, s, p, (int32_t)n);
    if (ok && s < v) { v = s; c = (int32_t)n; }
  }
  wave_min(v, c);
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = v; sc[threadIdx.x >> 6] = c; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < VF_PART / 64; ++w) take_min(v, c, sv[w], sc[w]);
    pval[(size_t)p * nparts + blockIdx.x] = v;
    pidx[(size_t)p * nparts + blockIdx.x] = c;
  }
}

// Final scan per group of candidates over the partial minima.
__global__ __launch_bounds__(64) void k_argmin_groups(const float *pval, const int32_t *pidx, int nparts,
                                                      int parts_per_group, int32_t *best_idx, float *best_val) {
  const int g = blockIdx.x;
  const int lo = g * parts_per_group;
  int hi = lo + parts_per_group;
  if (hi > nparts) hi = nparts;
  float v = __builtin_inff();
  int32_t c = -1;
  for (int p = lo + (int)threadIdx.x; p < hi; p += 64) take_min(v, c, pval[p], pidx[p]);
  wave_min(v, c);
  if (threadIdx.x == 0) {
    if (best_idx) best_idx[g] = c;
    if (best_val) best_val[g] = v;
  }
}

// --------------------------------------------------------------- bf16 MLP

struct MlpDev {
  int L;                 // weight layers; layer L-1 maps to the scalar value
  int dims[8];
  const uint16_t *w_pack;
  size_t pack_off[8];
  const float *aux;      // biases of every layer, then the last layer's vector
  size_t bias_off[8];
  size_t wl_off;
};

// Repack W[N][K] (fp32, row-major) into MFMA A-fragment order, rounded to bf16:
// out[tile][kstep][lane][e] = W[tile*32 + lane%32][kstep*16 + 8*(lane/32) + e].
__global__ __launch_bounds__(256) void k_pack_a(const float *W, int N, int K, uint16_t *out) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)N * K) return;
  int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  size_t rest = i >> 9;
  int ksteps = K / 16;
  int s = (int)(rest % ksteps), tile = (int)(rest / ksteps);
  int row = tile * 32 + (lane & 31), k = s * 16 + 8 * (lane >> 5) + e;
  out[i] = (uint16_t)bf16_bits(W[(size_t)row * K + k]);
}

__global__ __launch_bounds__(256) void k_copy_f32(const float *src, float *dst, size_t n, int round_bf16) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = round_bf16 ? bf16_val(src[i]) : src[i];
}

// The whole MLP for a tile of NC candidates.  8 waves; wave w owns the output row
// tiles w, w+8, ... (at most RT of them) of every hidden layer and all NC/32 candidate
// column tiles.  The weight fragments of a wave form one stream over all layers; a
// ring of PD k-steps of them is kept in flight so that L2 latency is hidden, also
// across the layer boundaries and behind the feature load.  The last hidden layer is
// never written back: its epilogue multiplies with the output vector directly.
template <int NC, int RT, int PD>
__global__ __launch_bounds__(512) void k_mlp_bf16(const int32_t *x, int64_t prob_stride, int64_t M, int64_t ld,
                                                  int use_valid_row, MlpDev md, int ks, float *scores,
                                                  int64_t ld_scores, float *pval, int32_t *pidx, int nparts,
                                                  NoiseArgs na) {
  constexpr int CT = NC / 32;
  constexpr int SEGS = 512 / NC;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *act = reinterpret_cast<uint16_t *>(smem);                   // [NC][ks]
  float *red = reinterpret_cast<float *>(smem + (size_t)NC * ks * 2);   // [8][NC]
  int32_t *okf = reinterpret_cast<int32_t *>(red + 8 * NC);             // [NC]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int p = blockIdx.y;
  const int64_t n0 = (int64_t)blockIdx.x * NC;
  const int32_t *xp = x + (size_t)p * prob_stride;
  const int NH = md.L - 1;  // hidden layers

  // ---- weight stream: prefetch cursor (layer, k-step) runs PD steps ahead
  uint4 ring[PD][RT];
  int pf_l = 0, pf_s = 0;
  auto prefetch = [&](int j) {
    if (pf_l < NH) {
      const int ksteps = md.dims[pf_l] / 16, ntiles = md.dims[pf_l + 1] / 32;
      const uint4 *Wp = reinterpret_cast<const uint4 *>(md.w_pack + md.pack_off[pf_l]);
#pragma unroll
      for (int r = 0; r < RT; ++r)
        if (w + r * 8 < ntiles) ring[j][r] = Wp[((size_t)(w + r * 8) * ksteps + pf_s) * 64 + lane];
      if (++pf_s == ksteps) { pf_s = 0; ++pf_l; }
    }
  };
#pragma unroll
  for (int j = 0; j < PD; ++j) prefetch(j);

  // ---- load: raw int32 [k][n] -> plog2 -> bf16 -> act[n][k]
  {
    const int F = md.dims[0];
    const int n = tid % NC;
    const bool inb = (n0 + n) < M;
    for (int k8 = tid / NC; k8 < F / 8; k8 += SEGS) {
      float h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int32_t raw = inb ? xp[(size_t)(k8 * 8 + e) * ld + n0 + n] : 0;
        h[e] = plog2_dev(raw);
        if (k8 == 2 && e == 0) okf[n] = inb && (!use_valid_row || raw != 0);
      }
      uint4 q;
      q.x = pack_bf16(h[0], h[1]); q.y = pack_bf16(h[2], h[3]);
      q.z = pack_bf16(h[4], h[5]); q.w = pack_bf16(h[6], h[7]);
      *reinterpret_cast<uint4 *>(act + (size_t)n * ks + k8 * 8) = q;
    }
  }
  __syncthreads();

  // ---- hidden layers
  float dot[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) dot[c] = 0.0f;
  for (int l = 0; l < NH; ++l) {
    const int K = md.dims[l], N = md.dims[l + 1];
    const int ntiles = N / 32, ksteps = K / 16;
    floatx16 acc[RT][CT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[r][c][j] = 0.0f;
    int mine = 0;
#pragma unroll
    for (int r = 0; r < RT; ++r) mine += (w + r * 8 < ntiles);
    const uint16_t *brow = act + (size_t)(lane & 31) * ks + 8 * (lane >> 5);
    for (int s0 = 0; s0 < ksteps; s0 += PD) {  // ksteps is a multiple of PD (host checks)
#pragma unroll
      for (int j = 0; j < PD; ++j) {
        uint4 a[RT], b[CT];
#pragma unroll
        for (int r = 0; r < RT; ++r) a[r] = ring[j][r];
        prefetch(j);
        if (mine > 0) {
#pragma unroll
          for (int c = 0; c < CT; ++c)
            b[c] = *reinterpret_cast<const uint4 *>(brow + (size_t)c * 32 * ks + (s0 + j) * 16);
#pragma unroll
          for (int r = 0; r < RT; ++r)
            if (r < mine) {
#pragma unroll
              for (int c = 0; c < CT; ++c)
                acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, a[r]), __builtin_bit_cast(bf16x8, b[c]), acc[r][c], 0, 0, 0);
            }
        }
      }
    }
    const float *bias = md.aux + md.bias_off[l];
    if (l < NH - 1) {
      __syncthreads();  // every wave has read the layer's input: it can be overwritten
#pragma unroll
      for (int r = 0; r < RT; ++r)
        if (r < mine) {
          const int mbase = (w + r * 8) * 32 + 4 * (lane >> 5);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 bv = *reinterpret_cast<const float4 *>(bias + mbase + 8 * g);
#pragma unroll
            for (int c = 0; c < CT; ++c) {
              uint2 q;
              q.x = pack_bf16(relu_bits(acc[r][c][4 * g + 0] + bv.x), relu_bits(acc[r][c][4 * g + 1] + bv.y));
              q.y = pack_bf16(relu_bits(acc[r][c][4 * g + 2] + bv.z), relu_bits(acc[r][c][4 * g + 3] + bv.w));
              *reinterpret_cast<uint2 *>(act + (size_t)(c * 32 + (lane & 31)) * ks + mbase + 8 * g) = q;
            }
          }
        }
      __syncthreads();
    } else {
      // last hidden layer: round to bf16 and multiply with the output vector at once
      const float *wl = md.aux + md.wl_off;
#pragma unroll
      for (int r = 0; r < RT; ++r)
        if (r < mine) {
          const int mbase = (w + r * 8) * 32 + 4 * (lane >> 5);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 bv = *reinterpret_cast<const float4 *>(bias + mbase + 8 * g);
            const float4 wv = *reinterpret_cast<const float4 *>(wl + mbase + 8 * g);
#pragma unroll
            for (int c = 0; c < CT; ++c) {
              uint32_t q0 = pack_bf16(relu_bits(acc[r][c][4 * g + 0] + bv.x), relu_bits(acc[r][c][4 * g + 1] + bv.y));
              uint32_t q1 = pack_bf16(relu_bits(acc[r][c][4 * g + 2] + bv.z), relu_bits(acc[r][c][4 * g + 3] + bv.w));
              float d = dot[c];
              d = fmaf(__uint_as_float(q0 << 16), wv.x, d);
              d = fmaf(__uint_as_float(q0 & 0xffff0000u), wv.y, d);
              d = fmaf(__uint_as_float(q1 << 16), wv.z, d);
              d = fmaf(__uint_as_float(q1 & 0xffff0000u), wv.w, d);
              dot[c] = d;
            }
          }
        }
    }
  }

  // ---- value: sum the partial dots of the two lane halves, then of the waves in order
  if (NH > 0) {
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      float v = dot[c] + __shfl_xor(dot[c], 32);
      if (lane < 32) red[w * NC + c * 32 + lane] = v;
    }
  } else {
    // no hidden layer: v = w_L . x + b_L straight from the input tile
    const int K = md.dims[0];
    const float *wl = md.aux + md.wl_off;
    const int n = tid % NC, seg = tid / NC;
    const int klen = K / SEGS;  // K is a multiple of 32, SEGS is 4 or 8
    float sum = 0.0f;
    const uint16_t *row = act + (size_t)n * ks + seg * klen;
    for (int k = 0; k < klen; k += 4) {
      uint2 q = *reinterpret_cast<const uint2 *>(row + k);
      const float4 wv = *reinterpret_cast<const float4 *>(wl + seg * klen + k);
      sum = fmaf(__uint_as_float(q.x << 16), wv.x, sum);
      sum = fmaf(__uint_as_float(q.x & 0xffff0000u), wv.y, sum);
      sum = fmaf(__uint_as_float(q.y << 16), wv.z, sum);
      sum = fmaf(__uint_as_float(q.y & 0xffff0000u), wv.w, sum);
    }
    red[seg * NC + n] = sum;
    for (int g = SEGS + seg; g < 8; g += SEGS) red[g * NC + n] = 0.0f;
  }
  __syncthreads();
  {
    float v = __builtin_inff();
    int32_t c = -1;
    if (tid < NC) {
      float s = md.aux[md.bias_off[md.L - 1]];
#pragma unroll
      for (int g = 0; g < 8; ++g) s += red[g * NC + tid];
      if (scores && (n0 + tid) < M) scores[(size_t)p * ld_scores + n0 + tid] = s;
      if (na.eps != 0.0f) s = add_noise(na, s, p, (int32_t)(n0 + tid));
      if (okf[tid] != 0 && s < v) { v = s; c = (int32_t)(n0 + tid); }
      wave_min(v, c);
    }
    if (NC > 64) {
      __shared__ float sv[NC / 64];
      __shared__ int32_t sc[NC / 64];
      if (tid < NC && lane == 0) { sv[w] = v; sc[w] = c; }
      __syncthreads();
      if (tid == 0) {
        for (int k = 1; k < NC / 64; ++k) take_min(v, c, sv[k], sc[k]);
        pval[(size_t)p * nparts + blockIdx.x] = v;
        pidx[(size_t)p * nparts + blockIdx.x] = c;
      }
    } else if (tid == 0) {
      pval[(size_t)p * nparts + blockIdx.x] = v;
      pidx[(size_t)p * nparts + blockIdx.x] = c;
    }
  }
}

// ------------------------------------------------- bf16 MLP, uniform hidden width


// Stream order for k_mlp_fast: wave w's fragments of all hidden layers back to back,
// out[w][step][r][lane][e] with step running over (layer, k step) and row tile
// w + 8 r; `pad` zero steps follow so that the prefetch never leaves the buffer.
__global__ __launch_bounds__(256) void k_pack_stream(const float *blob, vf_fast_dev md, int RT, int steps_total,
                                                     int pad, uint16_t *out) {
  // of the first layer only md.k0 k-steps are packed, starting with step md.k0ofs
  const size_t per_wave = (size_t)(steps_total + pad) * RT * 512;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= per_wave * 8) return;
  const int w = (int)(i / per_wave);
  size_t q = i % per_wave;
  const int e = (int)(q & 7), lane = (int)((q >> 3) & 63);
  q >>= 9;
  const int r = (int)(q % RT);
  int step = (int)(q / RT);
  uint16_t v = 0;
  if (step < steps_total) {
    size_t off = 0;
    for (int l = 0; l < md.L - 1; ++l) {
      const int K = md.dims[l], N = md.dims[l + 1], ksteps = l == 0 ? md.k0 : K / 16;
      if (step < ksteps) {
        const int kstep = l == 0 ? step + md.k0ofs : step;
        const int row = (w + 8 * r) * 32 + (lane & 31), k = kstep * 16 + 8 * (lane >> 5) + e;
        v = (uint16_t)bf16_bits(blob[off + (size_t)row * K + k]);
        break;
      }
      step -= ksteps;
      off += (size_t)K * N + N;
    }
  }
  out[i] = v;
}

// Fused MLP for hidden layers of exactly 256*RT units: every wave owns RT row tiles
// of every layer, so the main loop has no per-wave conditions; the weight stream of a
// wave is contiguous over all layers and is prefetched PD k-steps ahead without any
// branch; the activation fragments are read one k-step ahead.
//
// GEN = false: the tile's features are read from x (raw int32, feature-major).
// GEN = true: the tile's candidates are enumerated and featurized right here from
// the scheduling tables of problem blockIdx.y (x is not used): the features go
// straight into LDS as normalised bf16 and never touch HBM.  Of the network's input rows
// only 16..55 and 59 depend on the candidate: the product of the first layer with all the
// others (the intrinsic block, the context rows, with 256 inputs the neighbour stages) is
// computed once per decision and enters as the accumulators' starting value (fold_bias), and
// the candidates' contraction runs over rows 16..63 (three k-steps) with zeros in the shared
// rows among them.
struct GenArgs {
  const uint32_t *decpack;  // [problem][VF_DECPACK_DWORDS], built for the stage being decided
  unsigned long long *stat; // nullable: [0] += ids pushed through the network, [1] += valid ones
  // Chained layers (prev_stage >= 0): the launch for stage i first takes the decision of stage
  // i - 1 itself.  decpack is then the context of stage i - 1, pval_prev / pidx_prev its partial
  // minima [problem][nparts]; every workgroup reduces them, evaluates the winner and builds the
  // context of stage i from the tables and the winner's rows (Algorithm 1's s_{i-1} := s and the
  // next CandidateActions in one place); the workgroup that has a problem's first tile also
  // writes the winner to the tables and the new context to decpack_out, for the launch after.
  int prev_stage;
  const float *pval_prev;
  const int32_t *pidx_prev;
  uint32_t *decpack_out;
  Tables t;
};

// ONE (with GEN): the network has a single hidden layer.
// CHAIN (with GEN): the launch can also take the decision of the stage before (GenArgs::prev_stage).
template <int NC, int RT, int PD, bool GEN, bool ONE = false, bool CHAIN = false>
__global__ __launch_bounds__(512) void k_mlp_fast(const int32_t *x, int64_t prob_stride, int64_t M, int64_t ld,
                                                  int use_valid_row, vf_fast_dev md, int ks, float *scores,
                                                  int64_t ld_scores, float *pval, int32_t *pidx, int nparts,
                                                  int nprob, GenArgs ga, NoiseArgs na) {
  constexpr int CT = NC / 32;
  constexpr int SEGS = 512 / NC;
  constexpr int ROT = GEN ? VF_K0_OWN % PD : 0;  // ring slot of the first k-step behind the first layer
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *act = reinterpret_cast<uint16_t *>(smem);                   // [NC][ks]
  float *red = reinterpret_cast<float *>(smem + (size_t)NC * ks * 2);   // [8][NC]
  int32_t *okf = reinterpret_cast<int32_t *>(red + 8 * NC);             // [NC]
  float *auxs = reinterpret_cast<float *>(okf + NC);                    // [naux] biases, output vector
  float *b1s = auxs + ((md.naux + 3) & ~3);                             // [dims[1]] folded first-layer bias (GEN)
  __shared__ DecPack pk;
  int b1_p = -1;
  // (chained layers only)
  __shared__ DecPack pk_next;
  __shared__ DecScratch dscr;
  __shared__ EvalTabs tabs;
  __shared__ int32_t fresh_cf[64], fresh_st[16], fresh_sums[3], win_c;
  __shared__ float win_v;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int NH = md.L - 1;

  // ---- once per workgroup: the small fp32 vectors into LDS, the weight ring primed
  {
    float auxv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) auxv[q] = (tid + q * 512 < md.naux) ? md.aux[tid + q * 512] : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (tid + q * 512 < md.naux) auxs[tid + q * 512] = auxv[q];
    for (int i = tid + 2048; i < md.naux; i += 512) auxs[i] = md.aux[i];
  }
  const __amdgpu_buffer_rsrc_t ws = stream_rsrc(md.w_stream + (size_t)w * md.wave_stride);
  const int voff = 16 * lane;
  int wstep = PD;
  uint4 ring[PD][RT];
#pragma unroll
  for (int j = 0; j < PD; ++j)
#pragma unroll
    for (int r = 0; r < RT; ++r) ring[j][r] = stream_load(ws, voff, j * RT + r);

  // ---- persistent loop: this workgroup's share of the (problem, tile) pairs, in
  // problem-major order so that consecutive tiles mostly share the decision context
  const int T = nparts * nprob;
  const int t_begin = (int)((int64_t)blockIdx.x * T / gridDim.x);
  const int t_end = (int)((int64_t)(blockIdx.x + 1) * T / gridDim.x);
  int cur_p = -1;
  for (int t = t_begin; t < t_end; ++t) {
  const int p = t / nparts;
  const int64_t n0 = (int64_t)(t - p * nparts) * NC;
  const int32_t *xp = x + (size_t)p * prob_stride;
  if (GEN && p != cur_p) {
    if (tid < VF_DECPACK_DWORDS)
      reinterpret_cast<uint32_t *>(&pk)[tid] = ga.decpack[(size_t)p * VF_DECPACK_DWORDS + tid];
    cur_p = p;
    if (CHAIN && ga.prev_stage >= 0) {
      // ---- the decision of the stage before, then this stage's context
      float v = __builtin_inff();
      int32_t c = -1;
      if (w == 1) {  // (wave 1: wave 0 has the larger share of the context's fetch in front of it)
        for (int q = lane; q < nparts; q += 64) {
          const float pv = ga.pval_prev[(size_t)p * nparts + q];
          const int32_t pi = ga.pidx_prev[(size_t)p * nparts + q];
          if (pi >= 0 && (pv < v || (pv == v && (c < 0 || pi < c)))) { v = pv; c = pi; }
        }
        for (int off = 32; off > 0; off >>= 1) {
          const float ov = __shfl_down(v, off);
          const int32_t oc = __shfl_down(c, off);
          if (oc >= 0 && (ov < v || (ov == v && (c < 0 || oc < c)))) { v = ov; c = oc; }
        }
        if (lane == 0) { win_v = v; win_c = c; }
      }
      // what this stage's context takes from memory does not depend on the winner (the rows of
      // the stage before are left out): both rounds of fetches are under way while one thread
      // evaluates the winner
      dec_fetch_rows(pk_next.d, pk_next.sp, dscr, ga.t, p, ga.prev_stage + 1, ga.prev_stage);
      __syncthreads();  // the context of the stage before has arrived
      fill_evaltabs(tabs, pk.d, pk.sp, 64);
      dec_fetch_anchor(pk_next.d, dscr, ga.t, p, ga.prev_stage + 1, ga.prev_stage);
      __syncthreads();
      const bool writes = (int)((int64_t)p * nparts) >= t_begin;  // this workgroup has the problem's first tile
      if (tid == 0)
        commit_winner_fresh(ga.t, pk.d, pk.sp, p, ga.prev_stage, win_c, win_v, (uint32_t)M, tabs, writes, fresh_cf, fresh_st,
                            fresh_sums);
      __syncthreads();
      FreshRows fr;
      fr.stage = ga.prev_stage; fr.cf = fresh_cf; fr.st = fresh_st;
      fr.pm = fresh_sums[0]; fr.pb = fresh_sums[1]; fr.alive = fresh_sums[2];
      dec_finish(pk_next.d, pk_next.sp, dscr, ga.prev_stage + 1, fr);
      for (int q = tid; q < VF_STAT_WORDS; q += 512) pk_next.stat[q] = stat_word(pk_next.d, q);
      __syncthreads();
      {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&pk_next);
        const int used = (int)((sizeof(Dec) + sizeof(vf_space)) / 4 + VF_STAT_WORDS);
        if (tid < VF_DECPACK_DWORDS) {
          const uint32_t wv = tid < used ? src[tid] : 0u;
          reinterpret_cast<uint32_t *>(&pk)[tid] = wv;
          if (writes) ga.decpack_out[(size_t)p * VF_DECPACK_DWORDS + tid] = wv;
        }
      }
    }
  }
  __syncthreads();

  if (GEN) {
    // A tile none of whose ids can be valid is decided without the network.  For many
    // stages whole compute_at levels are closed, and that digit is the most significant
    // but one, so such ids come in runs much longer than a tile.
    const int64_t nend = (n0 + NC < M) ? n0 + NC : M;
    if (range_closed(pk.d, pk.sp, (uint32_t)n0, (uint32_t)(nend > n0 ? nend : n0))) {
      if (scores && tid < NC && (n0 + tid) < ld_scores) scores[(size_t)p * ld_scores + n0 + tid] = __builtin_inff();
      if (tid == 0) {
        pval[(size_t)t] = __builtin_inff();
        pidx[(size_t)t] = -1;
      }
      __syncthreads();  // the next tile may bring another problem's context
      continue;
    }
    if (b1_p != p) {
      fold_bias<RT>(stream_rsrc(md.w_full + (size_t)w * md.wave_stride_full), pk.stat, md.dims[0] == 256, w, lane,
                    auxs + md.bias_off[0], b1s);
      b1_p = p;
    }
    // ---- enumerate + featurize the tile: thread n < NC owns candidate n0 + n
    const Dec &dctx = pk.d;
    const vf_space &sp = pk.sp;
    // four threads per candidate, each producing part of the rows 16..63: the parts a
    // thread does not store are dead code in its copy of the evaluation
    {
      const int n = tid % NC, part = tid / NC;
      const bool inb = (n0 + n) < M;
      const uint32_t cid = (uint32_t)(n0 + n);
      int32_t core[64];
      uint32_t dec;
      // eight rows at a time: rows 16 + 8 q .. 23 + 8 q go to elements 8 q .. 8 q + 7 of the column
      auto put8 = [&](const int32_t *v, int q) {
        uint4 o;
        o.x = pack_bf16(plog2_dev(v[0]), plog2_dev(v[1]));
        o.y = pack_bf16(plog2_dev(v[2]), plog2_dev(v[3]));
        o.z = pack_bf16(plog2_dev(v[4]), plog2_dev(v[5]));
        o.w = pack_bf16(plog2_dev(v[6]), plog2_dev(v[7]));
        if (!inb) o = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4 *>(act + (size_t)n * ks + 8 * q) = o;
      };
      // the row groups are dealt out so that the four copies cost about the same
      if (part == 0) {
        // evaluated for padding ids too: core must be defined before it is packed
        const bool valid = eval_candidate<true>(dctx, sp, cid, dec, core);
        okf[n] = inb && valid;
        put8(core + 16, 0);
        put8(core + 24, 1);
      } else if (part == 1) {
        eval_candidate<true>(dctx, sp, cid, dec, core);
        put8(core + 32, 2);
        // rows 56..63: only row 59 is the candidate's own, the others are part of the bias
        uint4 o = make_uint4(0u, inb ? pack_bf16(0.0f, plog2_dev(core[59])) : 0u, 0u, 0u);
        *reinterpret_cast<uint4 *>(act + (size_t)n * ks + 40) = o;
      } else if (part == 2) {
        eval_candidate<true>(dctx, sp, cid, dec, core);
        put8(core + 40, 3);
      } else if (part == 3) {
        eval_candidate<true>(dctx, sp, cid, dec, core);
        put8(core + 48, 4);
      }
    }
  } else {
    // ---- load: raw int32 [k][n] -> plog2 -> bf16 -> act[n][k]; all loads of a pass
    // are issued before the first conversion
    const int F = md.dims[0];
    const int n = tid % NC;
    const bool inb = (n0 + n) < M;
    const int32_t *col = xp + n0 + n;
    constexpr int G = 2;  // groups of 8 features per pass
    for (int k8 = tid / NC; k8 < F / 8; k8 += SEGS * G) {
      int32_t raw[G][8];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int k = (k8 + g * SEGS) * 8 + e;
          raw[g][e] = (inb && k < F) ? col[(size_t)k * ld] : 0;
        }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int kk = k8 + g * SEGS;
        if (kk < F / 8) {
          if (kk == 2) okf[n] = inb && (!use_valid_row || raw[g][0] != 0);
          uint4 q;
          q.x = pack_bf16(plog2_dev(raw[g][0]), plog2_dev(raw[g][1]));
          q.y = pack_bf16(plog2_dev(raw[g][2]), plog2_dev(raw[g][3]));
          q.z = pack_bf16(plog2_dev(raw[g][4]), plog2_dev(raw[g][5]));
          q.w = pack_bf16(plog2_dev(raw[g][6]), plog2_dev(raw[g][7]));
          *reinterpret_cast<uint4 *>(act + (size_t)n * ks + kk * 8) = q;
        }
      }
    }
  }
  __syncthreads();

  float dot[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) dot[c] = 0.0f;
  const uint16_t *brow = act + (size_t)(lane & 31) * ks + 8 * (lane >> 5);
  // what follows a layer's contraction: the last hidden layer is rounded to bf16 and multiplied
  // with the output vector at once; any other one becomes the next layer's input - rounded to
  // bfloat16, ReLU on the pairs, the two lane halves trade their row groups so that every lane
  // writes 8 consecutive rows of its column at once
  auto finish_layer = [&](floatx16 (&acc)[RT][CT], bool lastl) __attribute__((always_inline)) {
    if (!lastl) {
      __syncthreads();  // every wave has read the layer's input: it can be overwritten
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
      __syncthreads();
    } else {
      // (the output vector sits in LDS as floats that are bfloat16 values: packing is exact)
      const float *wl = auxs + md.wl_off;
      output_dots_mfma<RT, CT>(acc, dot, [&](int u) { const float2 p = *reinterpret_cast<const float2 *>(wl + u); return pack_bf16(p.x, p.y); }, w, lane);
    }
  };
  if constexpr (GEN) {
    // the first layer over the candidates' own rows
    floatx16 acc[RT][CT], bv[RT];
    load_bias<RT>(bv, b1s, w, lane);
    contract_own_rows<RT, CT, PD, ONE>(acc, bv, ring, ws, voff, brow, 32 * ks);
    wstep = VF_K0_OWN + PD;
    finish_layer(acc, ONE);
  }
  for (int l = GEN ? 1 : 0; l < NH; ++l) {
    floatx16 acc[RT][CT], bv[RT];
    load_bias<RT>(bv, auxs + md.bias_off[l], w, lane);
    // (the last PD steps of a tile prefetch the first PD steps of the next one)
    contract_layer<RT, CT, PD, ROT>(acc, bv, ring, ws, wstep, voff, l == NH - 1, md.dims[l] / 16, brow, 32 * ks);
    finish_layer(acc, l == NH - 1);
  }
  if (!GEN) wstep = PD;

#pragma unroll
  for (int c = 0; c < CT; ++c)
    if (lane < 32) red[w * NC + c * 32 + lane] = dot[c];  // (lanes 0..31 hold the wave's part of the dot)
  __syncthreads();
  {
    float v = __builtin_inff();
    int32_t c = -1;
    if (tid < NC) {
      float s = auxs[md.bias_off[md.L - 1]];
#pragma unroll
      for (int g = 0; g < 8; ++g) s += red[g * NC + tid];
      // scores of a generated tile are masked: invalid candidates and padding read +inf
      if (scores && (GEN ? (n0 + tid) < ld_scores : (n0 + tid) < M))
        scores[(size_t)p * ld_scores + n0 + tid] = (GEN && okf[tid] == 0) ? __builtin_inff() : s;
      const int32_t colid = (int32_t)(n0 + tid);
      if (na.eps != 0.0f) s = add_noise(na, s, p, colid);
      if (okf[tid] != 0 && s < v) { v = s; c = colid; }
      wave_min(v, c);
      if (GEN && ga.stat) {
        const int nvalid = __popcll(__ballot(okf[tid] != 0));
        const int nin = __popcll(__ballot((n0 + tid) < M));
        if (lane == 0) {
          atomicAdd(&ga.stat[0], (unsigned long long)nin);
          atomicAdd(&ga.stat[1], (unsigned long long)nvalid);
        }
      }
    }
    if (NC > 64) {
      __shared__ float sv[NC / 64];
      __shared__ int32_t sc[NC / 64];
      if (tid < NC && lane == 0) { sv[w] = v; sc[w] = c; }
      __syncthreads();
      if (tid == 0) {
        for (int k = 1; k < NC / 64; ++k) take_min(v, c, sv[k], sc[k]);
        pval[(size_t)t] = v;
        pidx[(size_t)t] = c;
      }
    } else if (tid == 0) {
      pval[(size_t)t] = v;
      pidx[(size_t)t] = c;
    }
  }
  __syncthreads();  // the tile's LDS is free for the next one
  }
}

// --------------------------------------------------------------- bf16 LSTM

struct LstmDev {
  int F, H;
  const uint16_t *w_pack;  // [unit tile][k step][gate][lane][8]
  const float *aux;        // b_ih + b_hh [4H], head vector [H], head bias [1]
};

// [W_ih | W_hh] as one [4H][F+H] matrix in A-fragment order.  The wave that owns a
// tile of 32 hidden units reads, per k-step, the four gate fragments of that tile:
// they are adjacent, and the k-steps of one timestep form one contiguous stream.
__global__ __launch_bounds__(256) void k_pack_lstm(const float *Wih, const float *Whh, int F, int H,
                                                   uint16_t *out) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)4 * H * (F + H)) return;
  int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  size_t rest = i >> 9;
  int ksteps = (F + H) / 16;
  int g = (int)(rest % 4); rest /= 4;
  int s = (int)(rest % ksteps), u = (int)(rest / ksteps);
  int row = g * H + u * 32 + (lane & 31), k = s * 16 + 8 * (lane >> 5) + e;
  float v = k < F ? Wih[(size_t)row * F + k] : Whh[(size_t)row * H + (k - F)];
  out[i] = (uint16_t)bf16_bits(v);
}

__global__ __launch_bounds__(256) void k_lstm_aux(const float *bih, const float *bhh, const float *wh,
                                                  const float *bh, int H, float *aux) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < 4 * H) aux[i] = bih[i] + bhh[i];
  else if (i < 5 * H) aux[i] = bf16_val(wh[i - 4 * H]);
  else if (i == 5 * H) aux[i] = bh[0];
}


// One workgroup walks NC sequences through all T steps.  Wave w owns hidden units
// 32w..32w+31: the four gate row tiles of those units for every candidate column.
// Per step a wave has three pieces of work: the x_t part of the contraction (it does not
// depend on h_{t-1}), the h_{t-1} part, and the gates (5 exponentials and 3 reciprocals per
// cell, on the vector ALUs, about as long as both contractions together).  Per step: the x_t
// part, one barrier (h_{t-1} complete), the h_{t-1} part, the gates.  h is double-buffered
// in LDS so that h_t is written as it is produced; x_{t+1} is fetched a step ahead; the
// weight fragments of a timestep are one contiguous stream per wave, kept PD k-steps ahead
// in a register ring that wraps at the end of the step.
template <int NC, int XPT, int PD>
__global__ __launch_bounds__(512) void k_lstm_bf16(const uint16_t *x, int64_t M, int T, LstmDev md, int xld,
                                                   int hld, float *scores, float *pval, int32_t *pidx) {
  constexpr int CT = NC / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *xs = reinterpret_cast<uint16_t *>(smem);                  // [2][NC][xld]
  uint16_t *hs = xs + (size_t)2 * NC * xld;                          // [2][NC][hld]
  float *red = reinterpret_cast<float *>(hs + (size_t)2 * NC * hld);  // [8][NC]
  float *auxs = red + 8 * NC;                                         // [5H+1]

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int F = md.F, H = md.H;
  const int64_t n0 = (int64_t)blockIdx.x * NC;
  const int cpr = F / 8;                 // 16-byte chunks per sequence row
  const int nchunks = NC * cpr;          // <= 512 * XPT
  const int ksx = F / 16, ksh = H / 16, ksteps = ksx + ksh;
  const bool active = w < H / 32;
  const int wu = active ? w : 0;         // idle waves shadow tile 0 but never store
  // the wave's weight stream: base in scalar registers, 16 bytes per lane, fragment i at byte 1024 i
  const __amdgpu_buffer_rsrc_t ws = stream_rsrc(reinterpret_cast<const uint4 *>(md.w_pack) + (size_t)wu * ksteps * 4 * 64);
  const int voff = 16 * lane;
  int wstep = PD;  // the k-step of the timestep's stream that refills the next slot

  uint4 ring[PD][4];
#pragma unroll
  for (int j = 0; j < PD; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) ring[j][g] = stream_load(ws, voff, j * 4 + g);

  for (int i = tid; i < NC * hld; i += 512) reinterpret_cast<uint32_t *>(hs)[i] = 0u;  // both h buffers
  for (int i = tid; i < 8 * NC; i += 512) red[i] = 0.0f;
  for (int i = tid; i < 5 * H + 1; i += 512) auxs[i] = md.aux[i];

  uint4 xr[XPT];
  auto fetch = [&](int t) {
#pragma unroll
    for (int q = 0; q < XPT; ++q) {
      int ch = tid + q * 512;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (ch < nchunks && t < T) {
        int n = ch / cpr, kc = ch % cpr;
        if (n0 + n < M) v = *reinterpret_cast<const uint4 *>(x + ((size_t)(n0 + n) * T + t) * F + kc * 8);
      }
      xr[q] = v;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int q = 0; q < XPT; ++q) {
      int ch = tid + q * 512;
      if (ch < nchunks) {
        int n = ch / cpr, kc = ch % cpr;
        *reinterpret_cast<uint4 *>(xs + ((size_t)buf * NC + n) * xld + kc * 8) = xr[q];
      }
    }
  };

  floatx16 cst[CT];
  float vsum[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    vsum[c] = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) cst[c][j] = 0.0f;
  }

  const float *bias = auxs, *wh = auxs + 4 * H;
  const int rowoff = (lane & 31), koff = 8 * (lane >> 5);
  floatx16 acc[4][CT];
  // firstc: the timestep's first round - its first k-step starts the accumulators: the products of
  // a gate's row tile with every column tile take the gate's bias as their addend (gate by gate,
  // so that one bias vector is in registers at a time), and no accumulator is filled beforehand
  auto kloop = [&](const uint16_t *src, int ld, int nsteps, bool last_part, auto firstc) __attribute__((always_inline)) {
    constexpr bool first = decltype(firstc)::value;
    const uint16_t *brow = src + (size_t)rowoff * ld + koff;
    uint4 bcur[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) bcur[c] = *reinterpret_cast<const uint4 *>(brow + (size_t)c * 32 * ld);
    // (nothing but the ring's loads in flight at the loop's entry: the compiler then waits for
    // the oldest weight fragment only, not for all of them at the top of every round)
    __builtin_amdgcn_s_waitcnt(0x0070);
    auto round = [&](int s0, auto startc) __attribute__((always_inline)) {
      constexpr bool starts = decltype(startc)::value;
      if (last_part && s0 + PD >= nsteps) wstep = 0;  // wrap: next timestep's first fragments
#pragma unroll
      for (int j = 0; j < PD; ++j) {
        if constexpr (starts) {
          if (j == 0) {
            // (read afresh every timestep: kept in registers across the steps, the four bias
            // vectors would take 64 of them)
            int boff = wu * 32 + 4 * (lane >> 5);
            asm volatile("" : "+v"(boff));
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
        // that reads it: a column's activation fragment with the next k-step's, a weight
        // fragment with the one PD k-steps ahead
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
    int s0 = 0;
    if constexpr (first) { round(0, vf_tag<true>{}); s0 = PD; }
    for (; s0 < nsteps; s0 += PD) round(s0, vf_tag<false>{});
  };
  // gates and cell update of step t from the accumulators; h_t goes to the other h buffer
  auto gates = [&](int t) __attribute__((always_inline)) {
    uint16_t *hout = hs + (size_t)((t + 1) & 1) * NC * hld;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 whv = *reinterpret_cast<const float4 *>(wh + wu * 32 + 4 * (lane >> 5) + 8 * q);
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
          *reinterpret_cast<uint2 *>(hout + (size_t)(c * 32 + (lane & 31)) * hld + w * 32 + 8 * q + 4 * (lane >> 5)) = pkd;
        }
      }
    }
  };

  fetch(0);
  stash(0);
  fetch(1);
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    // x_{t+1} (fetched during the previous step) goes to the buffer last read at t-1
    stash((t + 1) & 1);
    fetch(t + 2);
    kloop(xs + (size_t)(t & 1) * NC * xld, xld, ksx, false, vf_tag<true>{});
    __syncthreads();  // h_{t-1} is complete; x_{t+1} is visible for the next step
    kloop(hs + (size_t)(t & 1) * NC * hld, hld, ksh, true, vf_tag<false>{});
    gates(t);
  }

  // v = sum_t (w . h_t + b): add the two lane halves, then the waves in order
  if (active) {
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      float v = vsum[c] + __shfl_xor(vsum[c], 32);
      if (lane < 32) red[w * NC + c * 32 + lane] = v;
    }
  }
  __syncthreads();
  {
    float v = __builtin_inff();
    int32_t cbest = -1;
    if (tid < NC) {
      float s = (float)T * auxs[5 * H];
#pragma unroll
      for (int k = 0; k < 8; ++k) s += red[k * NC + tid];
      const bool inb = (n0 + tid) < M;
      if (scores && inb) scores[n0 + tid] = s;
      if (inb && s < v) { v = s; cbest = (int32_t)(n0 + tid); }
      wave_min(v, cbest);
    }
    if (NC > 64) {
      __shared__ float sv[NC / 64];
      __shared__ int32_t sc[NC / 64];
      if (tid < NC && lane == 0) { sv[w] = v; sc[w] = cbest; }
      __syncthreads();
      if (tid == 0) {
        for (int k = 1; k < NC / 64; ++k) take_min(v, cbest, sv[k], sc[k]);
        pval[blockIdx.x] = v; pidx[blockIdx.x] = cbest;
      }
    } else if (tid == 0) {
      pval[blockIdx.x] = v; pidx[blockIdx.x] = cbest;
    }
  }
}

template <typename T>
int grow(vf_ctx *c, T *&p, size_t &have, size_t want) {
  if (want <= have) return VF_OK;
  if (p) { VF_HIP(c, hipStreamSynchronize(c->stream)); VF_HIP(c, hipFree(p)); p = nullptr; have = 0; }
  void *q = nullptr;
  if (hipMalloc(&q, want * sizeof(T)) != hipSuccess) { (void)hipGetLastError(); return VF_ENOMEM; }
  p = (T *)q; have = want;
  return VF_OK;
}

}  // namespace

int vfk_static_parts(vf_ctx *c, vf_partbuf *out) {
  // address of this device's copy of the array, asked for once per device with that device
  // current (the callers hold a guard on c->device)
  constexpr int MAXDEV = 64;
  static std::mutex mu;
  static void *dev_ptr[MAXDEV] = {nullptr};
  if (c->device < 0 || c->device >= MAXDEV) return VF_EINVAL;
  void *p = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_ptr[c->device]) {
      void *q = nullptr;
      const hipError_t e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !q) {
        (void)hipGetLastError();
        c->last_hip = (int)e;
        return VF_EHIP;
      }
      dev_ptr[c->device] = q;
    }
    p = dev_ptr[c->device];
  }
  out->val = reinterpret_cast<float *>(p);
  out->idx = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(p) + (size_t)VF_STATIC_PARTS * 4);
  out->cap = VF_STATIC_PARTS;
  return VF_OK;
}

int vfk_ensure_parts(vf_ctx *c, size_t n) {
  if (n <= c->part_elems) return VF_OK;
  size_t h1 = c->part_elems, h2 = c->part_elems;
  int rc = grow(c, c->d_pval, h1, n);
  if (rc != VF_OK) return rc;
  rc = grow(c, c->d_pidx, h2, n);
  if (rc != VF_OK) return rc;
  c->part_elems = n;
  return VF_OK;
}

void vfk_free_model(vf_ctx *c) {
  vfk_seq_free(c);
  if (c->pm.w_f32) (void)hipFree(c->pm.w_f32);
  if (c->pm.w_f32t) (void)hipFree(c->pm.w_f32t);
  if (c->pm.w_pack) (void)hipFree(c->pm.w_pack);
  if (c->pm.w_stream) (void)hipFree(c->pm.w_stream);
  if (c->pm.w_stream_fold) (void)hipFree(c->pm.w_stream_fold);
  if (c->pm.w_seqT) (void)hipFree(c->pm.w_seqT);
  if (c->pm.aux) (void)hipFree(c->pm.aux);
  c->pm = vf_packed_model();
}

int vfk_pack_model(vf_ctx *c, const float *wdev) {
  const vf_model &m = c->model;
  vf_packed_model &pm = c->pm;
  hipStream_t st = c->stream;
  auto blocks = [](size_t n) { return dim3((unsigned)((n + 255) / 256)); };
  if (m.kind == VF_MLP && m.dtype == VF_FP32) {
    size_t n = 0;
    for (int l = 0; l < m.n_layers; ++l) n += (size_t)m.dims[l] * m.dims[l + 1] + m.dims[l + 1];
    VF_HIP(c, hipMalloc((void **)&pm.w_f32, n * sizeof(float)));
    pm.n_floats = n;
    hipLaunchKernelGGL(k_copy_f32, blocks(n), dim3(256), 0, st, wdev, pm.w_f32, n, 0);
    VF_HIP(c, hipGetLastError());
    size_t nt = 0;
    for (int l = 0; l < m.n_layers; ++l) nt += (size_t)m.dims[l] * ((m.dims[l + 1] + 15) / 16 * 16);
    VF_HIP(c, hipMalloc((void **)&pm.w_f32t, nt * sizeof(float)));
    const float *src = wdev;
    float *dst = pm.w_f32t;
    for (int l = 0; l < m.n_layers; ++l) {
      const int K = m.dims[l], N = m.dims[l + 1], Npad = (N + 15) / 16 * 16;
      hipLaunchKernelGGL(k_transpose_f32, blocks((size_t)K * Npad), dim3(256), 0, st, src, K, N, Npad, dst);
      VF_HIP(c, hipGetLastError());
      src += (size_t)K * N + N;
      dst += (size_t)K * Npad;
    }
    return VF_OK;
  }
  if (m.kind == VF_MLP) {
    const int L = m.n_layers;
    size_t npack = 0, naux = 0;
    for (int l = 0; l < L; ++l) {
      if (l < L - 1) { pm.pack_off[l] = npack; npack += (size_t)m.dims[l] * m.dims[l + 1]; }
      pm.aux_off[l] = naux; naux += m.dims[l + 1];
    }
    naux = (naux + 3) / 4 * 4;  // keep the last layer's vector 16-byte aligned
    size_t wl_off = naux;
    naux += m.dims[L - 1];
    pm.aux_off[7] = wl_off;
    if (npack) VF_HIP(c, hipMalloc((void **)&pm.w_pack, npack * sizeof(uint16_t)));
    VF_HIP(c, hipMalloc((void **)&pm.aux, naux * sizeof(float)));
    size_t off = 0;
    for (int l = 0; l < L; ++l) {
      const int K = m.dims[l], N = m.dims[l + 1];
      const float *W = wdev + off, *b = W + (size_t)K * N;
      if (l < L - 1) {
        hipLaunchKernelGGL(k_pack_a, blocks((size_t)K * N), dim3(256), 0, st, W, N, K, pm.w_pack + pm.pack_off[l]);
      } else {
        hipLaunchKernelGGL(k_copy_f32, blocks((size_t)K), dim3(256), 0, st, W, pm.aux + wl_off, (size_t)K, 1);
      }
      VF_HIP(c, hipGetLastError());
      hipLaunchKernelGGL(k_copy_f32, blocks((size_t)N), dim3(256), 0, st, b, pm.aux + pm.aux_off[l], (size_t)N, 0);
      VF_HIP(c, hipGetLastError());
      off += (size_t)K * N + N;
    }
    // uniform hidden width 512 or 1024 with k-step counts that are multiples of 4 (the
    // deepest weight ring): pack the per-wave fragment stream for k_mlp_fast as well
    int rt = 0;
    if (L >= 2) {
      rt = m.dims[1] / 256;
      if (rt != 2 && rt != 4) rt = 0;
      for (int l = 1; l < L; ++l) if (m.dims[l] != 256 * rt) rt = 0;
      for (int l = 0; l < L - 1; ++l) if ((m.dims[l] / 16) % 4 != 0) rt = 0;
    }
    if (rt) {
      int steps = 0;
      for (int l = 0; l < L - 1; ++l) steps += m.dims[l] / 16;
      const int pad = 8;
      const size_t per_wave = (size_t)(steps + pad) * rt * 512;
      VF_HIP(c, hipMalloc((void **)&pm.w_stream, per_wave * 8 * sizeof(uint16_t)));
      vf_fast_dev fd;
      fd.L = L;
      for (int l = 0; l < 8; ++l) fd.dims[l] = m.dims[l];
      fd.k0 = m.dims[0] / 16;
      fd.k0ofs = 0;
      hipLaunchKernelGGL(k_pack_stream, blocks(per_wave * 8), dim3(256), 0, st, wdev, fd, rt, steps, pad, pm.w_stream);
      VF_HIP(c, hipGetLastError());
      pm.wave_stride = per_wave / 8;
      pm.fast_rt = rt;
      if (m.dims[0] == 64 || m.dims[0] == 256) {
        // the input widths of the search's feature layouts: the same stream with the first layer
        // cut down to the k-steps of the rows that depend on the candidate (16..63), for the
        // scorers that generate their candidates (the other rows' weights are read from the
        // whole stream, once per decision)
        const int fsteps = steps - (m.dims[0] / 16 - VF_K0_OWN);
        const size_t per_wave_f = (size_t)(fsteps + pad) * rt * 512;
        VF_HIP(c, hipMalloc((void **)&pm.w_stream_fold, per_wave_f * 8 * sizeof(uint16_t)));
        fd.k0 = VF_K0_OWN;
        fd.k0ofs = 1;
        hipLaunchKernelGGL(k_pack_stream, blocks(per_wave_f * 8), dim3(256), 0, st, wdev, fd, rt, fsteps, pad,
                           pm.w_stream_fold);
        VF_HIP(c, hipGetLastError());
        pm.wave_stride_fold = per_wave_f / 8;
      }
    }
    return VF_OK;
  }
  // LSTM, bf16
  const int F = m.dims[0], H = m.dims[1];
  size_t npack = (size_t)4 * H * (F + H);
  {
    // the blob as it is, for the per-problem prefix recurrence of the wired form
    const size_t n = npack + (size_t)9 * H + 1;
    VF_HIP(c, hipMalloc((void **)&pm.w_f32, n * sizeof(float)));
    pm.n_floats = n;
    hipLaunchKernelGGL(k_copy_f32, blocks(n), dim3(256), 0, st, wdev, pm.w_f32, n, 0);
    VF_HIP(c, hipGetLastError());
  }
  VF_HIP(c, hipMalloc((void **)&pm.w_pack, npack * sizeof(uint16_t)));
  VF_HIP(c, hipMalloc((void **)&pm.aux, (size_t)(5 * H + 1) * sizeof(float)));
  const float *Wih = wdev, *Whh = Wih + (size_t)4 * H * F, *bih = Whh + (size_t)4 * H * H;
  const float *bhh = bih + 4 * H, *wh = bhh + 4 * H, *bh = wh + H;
  hipLaunchKernelGGL(k_pack_lstm, blocks(npack), dim3(256), 0, st, Wih, Whh, F, H, pm.w_pack);
  VF_HIP(c, hipGetLastError());
  hipLaunchKernelGGL(k_lstm_aux, blocks((size_t)5 * H + 1), dim3(256), 0, st, bih, bhh, wh, bh, H, pm.aux);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

static int score_mlp(vf_ctx *c, const int32_t *x, int64_t prob_stride, int nprob, int64_t M, int64_t ld,
                     int use_valid_row, float *scores, int64_t ld_scores, int *nparts_out, int gen_stage,
                     int noise_stage, const vf_partbuf *parts = nullptr);

int vfk_score_mlp(vf_ctx *c, const int32_t *x, int64_t prob_stride, int nprob, int64_t M, int64_t ld,
                  int use_valid_row, float *scores, int64_t ld_scores, int *nparts_out, int noise_stage,
                  const vf_partbuf *parts) {
  return score_mlp(c, x, prob_stride, nprob, M, ld, use_valid_row, scores, ld_scores, nparts_out, -1, noise_stage,
                   parts);
}

bool vfk_can_fuse_step(const vf_ctx *c) {
  return c->has_model && c->model.kind == VF_MLP && c->model.dtype == VF_BF16 && c->pm.fast_rt != 0 &&
         c->model.dims[0] == c->space.F;
}

int vfk_step_fused(vf_ctx *c, int stage, int *nparts_out) {
  return score_mlp(c, nullptr, 0, c->B, c->M, c->Mpad, 1, nullptr, 0, nparts_out, stage, stage);
}

// (the condition under which score_mlp takes tiles of 64 candidates for a generated step)
static bool narrow_step(const vf_ctx *c) {
  int maxw = 0, ncu = 256;
  for (int l = 0; l < c->model.n_layers; ++l) if (c->model.dims[l] > maxw) maxw = c->model.dims[l];
  (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device);
  return maxw <= 512 && c->pm.fast_rt && ((c->M + 127) / 128) * c->B * 2 <= ncu;
}

bool vfk_can_chain(const vf_ctx *c) { return vfk_can_fuse_step(c) && c->M > 0 && narrow_step(c); }

int vfk_greedy_chain(vf_ctx *c, int first, int last) {
  if (!vfk_can_chain(c) || first > last) return VF_ESTATE;
  c->chain_on = true;
  c->chain_prev = -1;
  c->chain_par = 0;  // the first launch reads the context that vfk_prepare leaves in the first buffer
  int nparts = 0, rc = VF_OK;
  for (int i = first; i <= last && rc == VF_OK; ++i) {
    rc = score_mlp(c, nullptr, 0, c->B, c->M, c->Mpad, 1, nullptr, 0, &nparts, i, i);
    c->chain_prev = i;
    c->chain_par ^= 1;
  }
  c->chain_on = false;
  c->dec_stage = -1;  // the first buffer holds whatever stage wrote it last
  if (rc != VF_OK) {
    // a launch could not be made: the tables hold some of the layers' decisions but not the
    // last one's - back to the state the call started from
    (void)vfk_rewind(c, first);
    return rc;
  }
  // the last layer's decision: its partial minima and its context are in the set / buffer written last
  const int par = c->chain_par ^ 1;
  const size_t nset = (size_t)nparts * c->B;
  return vfk_commit_from(c, last, nparts, c->d_pval + (size_t)par * nset, c->d_pidx + (size_t)par * nset,
                         par ? c->d_decpack2 : c->d_decpack);
}

namespace {
// masks the scores of invalid candidates (validity row of the feature matrix) and of
// the padding columns with +inf
__global__ __launch_bounds__(256) void k_mask_scores(float *scores, const int32_t *feat, int64_t feat_stride,
                                                     int64_t M, int64_t Mpad) {
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int p = blockIdx.y;
  if (n >= Mpad) return;
  const bool ok = n < M && feat[(size_t)p * feat_stride + (size_t)16 * Mpad + n] != 0;
  if (!ok) scores[(size_t)p * Mpad + n] = __builtin_inff();
}
}  // namespace

int vfk_step_scores(vf_ctx *c, int stage) {
  const size_t want = (size_t)c->B * c->Mpad;
  int rc = grow(c, c->d_scores, c->score_elems, want);
  if (rc != VF_OK) return rc;
  int nparts = 0;
  if (vfk_seq_model(c)) return vfk_seq_step(c, stage, c->d_scores, c->Mpad, -1, &nparts);
  if (vfk_can_fuse_step(c)) return score_mlp(c, nullptr, 0, c->B, c->M, c->Mpad, 1, c->d_scores, c->Mpad, &nparts, stage, -1);
  // general models: materialise the features, score, mask
  const size_t fwant = (size_t)c->B * c->space.F * c->Mpad;
  rc = grow(c, c->d_feat, c->feat_elems, fwant);
  if (rc != VF_OK) return rc;
  rc = vfk_featurize(c, stage, c->d_feat);
  if (rc != VF_OK) return rc;
  const int64_t fstride = (int64_t)c->space.F * c->Mpad;
  rc = score_mlp(c, c->d_feat, fstride, c->B, c->M, c->Mpad, 1, c->d_scores, c->Mpad, &nparts, -1, -1);
  if (rc != VF_OK) return rc;
  hipLaunchKernelGGL(k_mask_scores, dim3((unsigned)((c->Mpad + 255) / 256), (unsigned)c->B), dim3(256), 0, c->stream,
                     c->d_scores, c->d_feat, fstride, c->M, c->Mpad);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}

// The packed bf16 MLP as the fused kernels take it.  generating: the candidates' features are
// produced in the kernel, so the first layer is cut down to the rows that depend on the
// candidate (k-steps 1..3) and the other rows' weights are handed over separately (w_full).
// ks / NC (nullable): row stride of the activation tile in LDS, candidates per tile.
void vfk_fast_dev(const vf_ctx *c, bool generating, vf_fast_dev *fd, int *ks, int *NC) {
  const vf_model &m = c->model;
  const int L = m.n_layers;
  fd->L = L;
  for (int l = 0; l < 8; ++l) { fd->dims[l] = m.dims[l]; fd->bias_off[l] = c->pm.aux_off[l]; }
  fd->w_stream = reinterpret_cast<const uint4 *>(c->pm.w_stream);
  fd->wave_stride = c->pm.wave_stride; fd->aux = c->pm.aux; fd->wl_off = c->pm.aux_off[7];
  fd->naux = (int)(c->pm.aux_off[7] + m.dims[L - 1]);
  fd->k0 = m.dims[0] / 16;
  fd->k0ofs = 0;
  fd->w_full = nullptr;
  fd->wave_stride_full = 0;
  if (generating && c->pm.w_stream_fold) {
    fd->w_stream = reinterpret_cast<const uint4 *>(c->pm.w_stream_fold);
    fd->wave_stride = c->pm.wave_stride_fold;
    fd->k0 = VF_K0_OWN;
    fd->k0ofs = 1;
    fd->w_full = reinterpret_cast<const uint4 *>(c->pm.w_stream);
    fd->wave_stride_full = c->pm.wave_stride;
  }
  int maxw = 0;
  for (int l = 0; l < L; ++l) if (m.dims[l] > maxw) maxw = m.dims[l];
  if (ks) *ks = maxw + 8;
  if (NC) *NC = maxw > 512 ? 64 : 128;
}

static int score_mlp(vf_ctx *c, const int32_t *x, int64_t prob_stride, int nprob, int64_t M, int64_t ld,
                     int use_valid_row, float *scores, int64_t ld_scores, int *nparts_out, int gen_stage,
                     int noise_stage, const vf_partbuf *parts) {
  NoiseArgs na;
  na.eps = noise_stage >= 0 ? c->noise_eps : 0.0f;
  na.k0 = (uint32_t)c->noise_seed; na.k1 = (uint32_t)(c->noise_seed >> 32);
  na.stage = noise_stage; na.first_rollout = c->noise_first;
  const vf_model &m = c->model;
  const int L = m.n_layers;
  hipStream_t st = c->stream;
  if (m.dtype == VF_FP32) {
    if (parts) return VF_EINVAL;  // the layer-by-layer kernels keep whole activation matrices in scratch
    int maxh = 1;
    for (int l = 1; l <= L; ++l) if (m.dims[l] > maxh) maxh = m.dims[l];
    const size_t per_prob = (size_t)maxh * ld;
    size_t h0 = c->act_elems, h1 = c->act_elems;
    int rc = grow(c, c->d_act[0], h0, per_prob * nprob);
    if (rc == VF_OK) rc = grow(c, c->d_act[1], h1, per_prob * nprob);
    if (rc != VF_OK) return rc;
    c->act_elems = h0 < h1 ? h0 : h1;
    const int nparts = (int)((M + VF_PART - 1) / VF_PART);
    rc = vfk_ensure_parts(c, (size_t)nparts * nprob);
    if (rc != VF_OK) return rc;
    const float *wp = c->pm.w_f32;
    const float *wt = c->pm.w_f32t;
    const void *in = x;
    int64_t in_stride = prob_stride, ld_in = ld;
    const float *final_scores = nullptr;
    int64_t final_stride = 0;
    for (int l = 0; l < L; ++l) {
      const int K = m.dims[l], N = m.dims[l + 1], Npad = (N + 15) / 16 * 16;
      const float *b = wp + (size_t)K * N;
      float *out = c->d_act[l & 1];
      int64_t out_stride = (int64_t)per_prob, ld_out = ld;
      if (l == L - 1) {
        if (scores) { out = scores; out_stride = ld_scores; ld_out = ld_scores; }
        final_scores = out; final_stride = out_stride;
      }
      dim3 grid((unsigned)((M + 255) / 256), (unsigned)((N + 15) / 16), (unsigned)nprob);
      if (M > 0) {
        if (l == 0)
          hipLaunchKernelGGL(k_mlp_f32_layer<true>, grid, dim3(256), 0, st, in, in_stride, ld_in, wt, Npad, b, out,
                             out_stride, ld_out, K, N, M, (int)(l < L - 1));
        else
          hipLaunchKernelGGL(k_mlp_f32_layer<false>, grid, dim3(256), 0, st, in, in_stride, ld_in, wt, Npad, b, out,
                             out_stride, ld_out, K, N, M, (int)(l < L - 1));
        VF_HIP(c, hipGetLastError());
      }
      in = out; in_stride = out_stride; ld_in = ld_out;
      wp = b + N;
      wt += (size_t)K * Npad;
    }
    if (nparts > 0) {
      hipLaunchKernelGGL(k_argmin_parts, dim3((unsigned)nparts, (unsigned)nprob), dim3(VF_PART), 0, st,
                         final_scores, final_stride, use_valid_row ? x + (size_t)16 * ld : (const int32_t *)nullptr,
                         prob_stride, M, nparts, c->d_pval, c->d_pidx, na);
      VF_HIP(c, hipGetLastError());
    }
    *nparts_out = nparts;
    return VF_OK;
  }
  // bf16: one fused kernel
  int maxw = 0;
  for (int l = 0; l < L; ++l) if (m.dims[l] > maxw) maxw = m.dims[l];
  MlpDev md;
  md.L = L;
  for (int l = 0; l < 8; ++l) { md.dims[l] = m.dims[l]; md.pack_off[l] = c->pm.pack_off[l]; md.bias_off[l] = c->pm.aux_off[l]; }
  md.w_pack = c->pm.w_pack; md.aux = c->pm.aux; md.wl_off = c->pm.aux_off[7];
  const int ks = maxw + 8;
  const bool wide = maxw > 512;
  int ncu = 256;
  (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device);
  // A decision of a few pipelines has fewer tiles of 128 candidates than half the compute
  // units: then tiles of 64 spread the same work over twice as many of them, and the
  // contraction of a tile - most of the time a layer takes - is half as long.
  const bool narrow = !wide && gen_stage >= 0 && c->pm.fast_rt && ((M + 127) / 128) * nprob * 2 <= ncu;  // (see narrow_step)
  const int NC = (wide || narrow) ? 64 : 128;
  const int nparts = (int)((M + NC - 1) / NC);
  float *pval = nullptr;
  int32_t *pidx = nullptr;
  const bool chained = c->chain_on && narrow && !parts && nparts > 0;
  const size_t nset = (size_t)(nparts > 0 ? nparts : 1) * nprob;
  if (parts) {
    if (nset > parts->cap) return VF_EINVAL;
    pval = parts->val; pidx = parts->idx;
  } else {
    // (chained layers: two sets, the one being written and the one of the stage before)
    int rc = vfk_ensure_parts(c, chained ? 2 * nset : nset);
    if (rc != VF_OK) return rc;
    pval = c->d_pval + (chained ? (size_t)c->chain_par * nset : 0);
    pidx = c->d_pidx + (chained ? (size_t)c->chain_par * nset : 0);
  }
  const size_t smem = (size_t)NC * ks * 2 + (size_t)8 * NC * 4 + (size_t)NC * 4;
  if (nparts > 0 && c->pm.fast_rt) {
    vf_prof_scope prof(c, VF_PROF_SCORE);
    vf_fast_dev fd;
    vfk_fast_dev(c, gen_stage >= 0, &fd, nullptr, nullptr);
    size_t smem_fast = smem + (size_t)fd.naux * 4;
    if (fd.w_full) smem_fast = smem + (size_t)((fd.naux + 3) & ~3) * 4 + (size_t)m.dims[1] * 4;
    // persistent: at most one workgroup per CU, each walking its share of the tiles
    const int64_t tiles = (int64_t)nparts * nprob;
    dim3 grid((unsigned)(tiles < ncu ? tiles : ncu));
    void (*kern)(const int32_t *, int64_t, int64_t, int64_t, int, vf_fast_dev, int, float *, int64_t, float *, int32_t *, int,
                 int, GenArgs, NoiseArgs);
    GenArgs ga;
    ga.decpack = c->d_decpack;
    ga.stat = c->profiling ? c->d_stat : nullptr;
    ga.prev_stage = -1;
    ga.pval_prev = nullptr;
    ga.pidx_prev = nullptr;
    ga.decpack_out = nullptr;
    ga.t = tables_of(c);
    if (chained && c->chain_prev >= 0) {
      uint32_t *const buf[2] = {c->d_decpack, c->d_decpack2};
      ga.prev_stage = c->chain_prev;
      ga.pval_prev = c->d_pval + (size_t)(c->chain_par ^ 1) * nset;
      ga.pidx_prev = c->d_pidx + (size_t)(c->chain_par ^ 1) * nset;
      ga.decpack = buf[c->chain_par ^ 1];
      ga.decpack_out = buf[c->chain_par];
    }
    if (gen_stage >= 0) {
      if (ga.prev_stage < 0) {
        int rc2 = vfk_prepare(c, gen_stage);
        if (rc2 != VF_OK) return rc2;
      }
      if (L == 2)
        kern = wide ? k_mlp_fast<64, 4, 2, true, true> : narrow ? k_mlp_fast<64, 2, 4, true, true, true> : k_mlp_fast<128, 2, 4, true, true>;
      else
        kern = wide ? k_mlp_fast<64, 4, 2, true> : narrow ? k_mlp_fast<64, 2, 4, true, false, true> : k_mlp_fast<128, 2, 4, true>;
    } else {
      kern = wide ? k_mlp_fast<64, 4, 4, false> : k_mlp_fast<128, 2, 4, false>;
    }
    VF_HIP(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_fast));
    hipLaunchKernelGGL(kern, grid, dim3(512), smem_fast, st, x, prob_stride, M, ld, use_valid_row, fd, ks, scores,
                       ld_scores, pval, pidx, nparts, nprob, ga, na);
    VF_HIP(c, hipGetLastError());
  } else if (nparts > 0) {
    vf_prof_scope prof(c, VF_PROF_SCORE);
    dim3 grid((unsigned)nparts, (unsigned)nprob);
    void (*kern)(const int32_t *, int64_t, int64_t, int64_t, int, MlpDev, int, float *, int64_t, float *, int32_t *, int,
                 NoiseArgs);
    if (wide) kern = k_mlp_bf16<64, 4, 2>;
    else kern = k_mlp_bf16<128, 2, 2>;
    VF_HIP(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(kern, grid, dim3(512), smem, st, x, prob_stride, M, ld, use_valid_row, md, ks, scores,
                       ld_scores, pval, pidx, nparts, na);
    VF_HIP(c, hipGetLastError());
  }
  *nparts_out = nparts;
  return VF_OK;
}

int vfk_score_lstm(vf_ctx *c, const uint16_t *x, int64_t M, int T, float *scores, int *nparts_out,
                   const vf_partbuf *parts) {
  const vf_model &m = c->model;
  constexpr int NC = 64;
  LstmDev md;
  md.F = m.dims[0]; md.H = m.dims[1]; md.w_pack = c->pm.w_pack; md.aux = c->pm.aux;
  const int xld = md.F + 8, hld = md.H + 8;
  const int nparts = (int)((M + NC - 1) / NC);
  float *pval = nullptr;
  int32_t *pidx = nullptr;
  if (parts) {
    if ((size_t)(nparts > 0 ? nparts : 1) > parts->cap) return VF_EINVAL;
    pval = parts->val; pidx = parts->idx;
  } else {
    int rc = vfk_ensure_parts(c, (size_t)(nparts > 0 ? nparts : 1));
    if (rc != VF_OK) return rc;
    pval = c->d_pval; pidx = c->d_pidx;
  }
  const size_t smem = (size_t)2 * NC * xld * 2 + (size_t)2 * NC * hld * 2 + (size_t)8 * NC * 4 +
                      (size_t)(5 * md.H + 1) * 4;
  if (nparts > 0) {
    vf_prof_scope prof(c, VF_PROF_SCORE);
    // ring depth 2: F and H are multiples of 32, so both parts have an even number of
    // k-steps (depth 4 spills registers and measured slower)
    void (*kern)(const uint16_t *, int64_t, int, LstmDev, int, int, float *, float *, int32_t *) =
        md.F <= 128 ? k_lstm_bf16<NC, 2, 2> : k_lstm_bf16<NC, 4, 2>;
    VF_HIP(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(kern, dim3((unsigned)nparts), dim3(512), smem, c->stream, x, M, T, md, xld, hld, scores,
                       pval, pidx);
    VF_HIP(c, hipGetLastError());
  }
  *nparts_out = nparts;
  return VF_OK;
}

int vfk_argmin_groups(vf_ctx *c, int64_t M, int nparts, int parts_per_group, int ngroups, int32_t *best_idx,
                      float *best_val, const vf_partbuf *parts) {
  (void)M;
  hipLaunchKernelGGL(k_argmin_groups, dim3((unsigned)ngroups), dim3(64), 0, c->stream,
                     parts ? parts->val : c->d_pval, parts ? parts->idx : c->d_pidx, nparts,
                     parts_per_group, best_idx, best_val);
  VF_HIP(c, hipGetLastError());
  return VF_OK;
}
