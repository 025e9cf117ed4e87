// Small device helpers shared by the scoring kernels.  Included inside the anonymous
// namespace of each .hip file that needs them, after vf_sched_dev.h.
#ifndef VF_SCORE_DEV_H
#define VF_SCORE_DEV_H

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// float -> bfloat16 bits, round to nearest, ties to even
__device__ __forceinline__ uint32_t bf16_bits(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_val(float v) { return __uint_as_float(bf16_bits(v) << 16); }
__device__ __forceinline__ float relu_keep_nan(float v) { return v < 0.0f ? 0.0f : v; }

// ReLU on the bit pattern: negative values (sign bit set, including -0) become +0,
// everything else, NaN included, is kept
__device__ __forceinline__ float relu_bits(float v) {
  int32_t i = __float_as_int(v);
  return __int_as_float(i < 0 ? 0 : i);
}

typedef short vf_shortx2 __attribute__((ext_vector_type(2)));

// ReLU of a packed bfloat16 pair, on the bit patterns like relu_bits: a half with the sign
// bit set becomes +0 (rounding to bfloat16 keeps the sign, so the order of the two is free)
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t q) {
  const vf_shortx2 zero = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(vf_shortx2, q), zero));
}

// Lanes 0..31 hand their b to lanes 32..63 and take those lanes' a: afterwards a lane below
// 32 holds (its a, the a of lane + 32) and a lane from 32 up (the b of lane - 32, its b).
__device__ __forceinline__ void swap_halves(uint32_t &a, uint32_t &b) {
  const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}

// (value, id) ordering of the scan: smaller value first, then smaller id; id < 0 = none
__device__ __forceinline__ void take_min(float &v, int32_t &c, float ov, int32_t oc) {
  if (oc >= 0 && (ov < v || (ov == v && (c < 0 || oc < c)))) { v = ov; c = oc; }
}
// Minimum pair of a full wave, left in every lane.  Rows of 16 lanes reduce by data-parallel
// lane shifts (lane i takes lane i - n; a lane without a source keeps its own pair), the four
// row results are then read from lanes 15, 31, 47 and 63.  All 64 lanes must be active.
__device__ __forceinline__ void wave_min(float &v, int32_t &c) {
#define VF_ROW_SHR_MIN(ctrl)                                                                              \
  {                                                                                                       \
    const float ov = __int_as_float(                                                                      \
        __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, 0xf, 0xf, false));        \
    const int32_t oc = __builtin_amdgcn_update_dpp(c, c, ctrl, 0xf, 0xf, false);                          \
    take_min(v, c, ov, oc);                                                                               \
  }
  VF_ROW_SHR_MIN(0x111)
  VF_ROW_SHR_MIN(0x112)
  VF_ROW_SHR_MIN(0x114)
  VF_ROW_SHR_MIN(0x118)
#undef VF_ROW_SHR_MIN
  float rv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
  int32_t rc = __builtin_amdgcn_readlane(c, 15);
  take_min(rv, rc, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31)), __builtin_amdgcn_readlane(c, 31));
  take_min(rv, rc, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 47)), __builtin_amdgcn_readlane(c, 47));
  take_min(rv, rc, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63)), __builtin_amdgcn_readlane(c, 63));
  v = rv;
  c = rc;
}

// One cell of the recurrent network in fp32: gate pre-activations ai, af, ag, ao and the old cell
// state give the new cell state (returned through c) and the new hidden value (returned).
//   c' = sigma(af) c + sigma(ai) tanh(ag),   h' = sigma(ao) tanh(c')
// A product sigma(a) tanh(b) is one quotient (e^{2b} - 1) / ((1 + e^{2b}) (1 + e^{-a})): two
// exponentials and one reciprocal instead of two and two, which matters because these run at a
// quarter of the rate of ordinary instructions (8 instead of 10 per cell).  Exponents are cut
// off at 60 binary orders, where tanh is 1 and sigma is 0 to far below fp32 resolution, so that
// the product of the two denominators stays finite; a NaN passes the cut-off and comes out.
__device__ __forceinline__ float exp2_cut(float x) { return __builtin_amdgcn_exp2f(x > 60.0f ? 60.0f : x); }
__device__ __forceinline__ float sig_tanh(float a, float b) {
  constexpr float LOG2E = 1.44269504088896340736f;
  const float ea = exp2_cut(a * -LOG2E), eb = exp2_cut(b * (2.0f * LOG2E));
  return (eb - 1.0f) * __builtin_amdgcn_rcpf((1.0f + eb) * (1.0f + ea));
}
__device__ __forceinline__ float lstm_cell(float ai, float af, float ag, float ao, float &c) {
  constexpr float LOG2E = 1.44269504088896340736f;
  const float fg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(af * -LOG2E));
  const float cn = fg * c + sig_tanh(ai, ag);
  c = cn;
  return sig_tanh(ao, cn);
}

// ---- pieces of the fused bf16 MLP that the per-layer scorer and the whole-schedule kernel share

// k-steps (16 input rows each) of the first layer that a candidate's own rows 16..63 take
constexpr int VF_K0_OWN = 3;

// A wave's weight stream as a buffer: the base address sits in scalar registers, a lane adds
// its own 16 bytes (voff = 16 * lane) and the fragment's position comes as a scalar byte offset,
// so that no vector register holds an address and no vector instruction computes one.  Fragment
// i of the stream (64 lanes x 16 bytes) starts at byte 1024 * i.
typedef unsigned int vf_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_rsrc(const void *p) {
  // no stride, no bound that could clip (the callers stay inside the stream), raw 32-bit format
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, -1, 0x00020000);
}
__device__ __forceinline__ uint4 stream_load(__amdgpu_buffer_rsrc_t rs, int voff, int frag) {
  return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, frag * 1024, 0));
}

// The first layer's product with the input rows that all candidates of a decision share, once
// per decision: the same contraction as for the candidates, with the shared vector in every
// column of one column tile, over k-steps 0 and 3 of the whole first layer (rows 0..15, and
// rows 48..63 with the candidates' own rows zero) and, with 256 inputs, k-steps 4..15 (rows
// 64..255).  Column 0 of the result plus the layer's bias is what the candidates'
// accumulators start from.  wf: this wave's fragments of the whole stream; stat:
// DecPack::stat; wide: 256 input rows.  Every wave of the workgroup calls it for its RT row tiles.
template <int RT>
__device__ __forceinline__ void fold_bias(__amdgpu_buffer_rsrc_t wf, const uint32_t *stat, bool wide, int w, int lane,
                                          const float *bias_in, float *bias_out) {
  floatx16 fa[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int q = 0; q < 16; ++q) fa[r][q] = 0.0f;
  const int n = wide ? 14 : 2;
#pragma unroll 7
  for (int q = 0; q < n; ++q) {
    const int sk = q == 0 ? 0 : q + 2;  // k-step of the whole first layer: 0, 3, 4, 5, ...
    uint4 a[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) a[r] = stream_load(wf, 16 * lane, sk * RT + r);
    const uint32_t *xb = stat + 8 * q + 4 * (lane >> 5);
    uint4 bv;
    bv.x = xb[0]; bv.y = xb[1]; bv.z = xb[2]; bv.w = xb[3];
#pragma unroll
    for (int r = 0; r < RT; ++r)
      fa[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[r]), __builtin_bit_cast(bf16x8, bv),
                                                     fa[r], 0, 0, 0);
  }
  if ((lane & 31) == 0) {
#pragma unroll
    for (int r = 0; r < RT; ++r) {
      const int mbase = (w + r * 8) * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) bias_out[mbase + 8 * g + e] = bias_in[mbase + 8 * g + e] + fa[r][4 * g + e];
    }
  }
}

// The bias of a wave's output rows, as the accumulator of one column tile holds them (row tile r
// of the wave = rows (w + 8 r) * 32 ..; a lane has rows 4 (lane >> 5) + 8 g + 0..3 of it).  The
// contractions take it as the addend of a layer's first k-step, for every column tile alike, so
// that no accumulator has to be filled with it beforehand.
template <int RT>
__device__ __forceinline__ void load_bias(floatx16 (&bv)[RT], const float *bias, int w, int lane) {
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    const int mbase = (w + r * 8) * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *reinterpret_cast<const float4 *>(bias + mbase + 8 * g);
      bv[r][4 * g + 0] = v.x; bv[r][4 * g + 1] = v.y; bv[r][4 * g + 2] = v.z; bv[r][4 * g + 3] = v.w;
    }
  }
}

template <bool V>
struct vf_tag { static constexpr bool value = V; };

// The contraction of one layer for a wave: RT row tiles x CT column tiles of 32 x 32, weights
// (A operand) from a ring of PD k-steps of fragments in registers, activations (B operand) from
// LDS.  With at least as many column tiles as row tiles (the tile of 128 candidates) the products
// of a k-step go column by column, and every operand register is refilled in place right behind
// the last product that reads it: a column's activation fragment with that of
// the next k-step (one step past the end stays inside LDS), a weight fragment with the one PD
// k-steps ahead - so there is at most one memory instruction behind a product (two behind the
// last one), the loads of a k-step are spread evenly over it, no second set of fragment
// registers is needed, and only the oldest slot of the ring is ever waited for.
//
// ws: the wave's weight stream; k-step n of a tile (its layers' k-steps counted through) is
// fragments n * RT .. n * RT + RT - 1 of it and lives in ring slot n % PD; a layer that starts
// at step n0 passes ROT = n0 % PD and wstep = n0 + PD, the step that refills the first slot
// (advanced as the loop goes).  ksteps is a multiple of PD.  wrap: the last PD steps are a
// tile's last ones and refill their slots with the next tile's first PD steps (step m into slot m).
// bb: this lane's B operand base (column lane & 31 of column tile 0, k half lane >> 5), cstride:
// elements between column tiles; consecutive k-steps are 16 elements apart.  bv: the bias
// (load_bias): the accumulators come out of the first k-step as product + bias.
template <int RT, int CT, int PD, int ROT>
__device__ __forceinline__ void contract_layer(floatx16 (&acc)[RT][CT], const floatx16 (&bv)[RT], uint4 (&ring)[PD][RT],
                                               __amdgpu_buffer_rsrc_t ws, int &wstep, int voff, bool wrap, int ksteps,
                                               const uint16_t *bb, int cstride) {
  uint4 bcur[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) bcur[c] = *reinterpret_cast<const uint4 *>(bb + (size_t)c * cstride);
  // Nothing but this loop's own loads may be in flight when it starts: with a store to scratch
  // or a scalar load still counted, the compiler can no longer tell the order in which the
  // counters come down and waits for every load at the top of each round instead of for the
  // oldest one.  (vmcnt 0, lgkmcnt 0; the ring's loads were issued long before.)
  __builtin_amdgcn_s_waitcnt(0x0070);
  // one round of PD k-steps; the layer's first round apart, since its first step starts the accumulators
  auto round = [&](int s0, auto firstc) __attribute__((always_inline)) {
    constexpr bool first = decltype(firstc)::value;
    const bool last = wrap && s0 + PD >= ksteps;
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      const int slot = (ROT + j) % PD;
      const int frag = (last ? slot : wstep + j) * RT;
      if constexpr (RT <= CT) {
#pragma unroll
        for (int i = 0; i < RT * CT; ++i) {
          const int c = i / RT, r = i % RT;
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[slot][r]),
                                                             __builtin_bit_cast(bf16x8, bcur[c]),
                                                             (first && j == 0) ? bv[r] : acc[r][c], 0, 0, 0);
          if (r == RT - 1) bcur[c] = *reinterpret_cast<const uint4 *>(bb + (size_t)c * cstride + (s0 + j + 1) * 16);
          if (c == CT - 1) ring[slot][r] = stream_load(ws, voff, frag + r);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        // more row tiles than column tiles: row by row, the few activation fragments of the next
        // k-step in a second set of registers (measured: the better order for this shape)
        uint4 bnext[CT];
#pragma unroll
        for (int i = 0; i < RT * CT; ++i) {
          const int r = i / CT, c = i % CT;
          acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[slot][r]),
                                                             __builtin_bit_cast(bf16x8, bcur[c]),
                                                             (first && j == 0) ? bv[r] : acc[r][c], 0, 0, 0);
          if (i < CT) bnext[i] = *reinterpret_cast<const uint4 *>(bb + (size_t)i * cstride + (s0 + j + 1) * 16);
          if (c == CT - 1) ring[slot][r] = stream_load(ws, voff, frag + r);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = 0; c < CT; ++c) bcur[c] = bnext[c];
      }
    }
    wstep += PD;
  };
  round(0, vf_tag<true>{});
  for (int s0 = PD; s0 < ksteps; s0 += PD) round(s0, vf_tag<false>{});
}

// The output layer on the matrix core.  The last hidden layer is never written back: rounded
// to bfloat16 (ReLU on the packed pairs), a lane's 8 accumulator values of one half of a row tile
// (rows 16 s + 4 h + 0..3 and 16 s + 8 + 4 h + 0..3 of it, h = lane >> 5) are already what a B
// operand wants of a lane - column lane & 31, eight of a k-step's sixteen rows - up to the order of
// the rows inside the k-step, and that order is free as long as the A operand follows it.  A = the
// output vector's entries for those rows in row 0 of the tile (lanes 0 and 32), zeros elsewhere;
// row 0 of the product (accumulator element 0 of lanes 0..31) is the wave's part of the dot for
// column lane & 31, both lane halves' rows included.  wl2(u), u even: the output vector's entries
// for hidden units u and u + 1 as a packed bfloat16 pair.  dot[c] is valid in lanes 0..31.
template <int RT, int CT, typename WL>
__device__ __forceinline__ void output_dots_mfma(const floatx16 (&acc)[RT][CT], float (&dot)[CT], WL wl2, int w, int lane) {
  uint4 af[RT][2];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int base = (w + r * 8) * 32 + 16 * s2 + 4 * (lane >> 5);
      uint4 a;
      a.x = wl2(base + 0);
      a.y = wl2(base + 2);
      a.z = wl2(base + 8);
      a.w = wl2(base + 10);
      if ((lane & 31) != 0) a = make_uint4(0u, 0u, 0u, 0u);
      af[r][s2] = a;
    }
  auto bfrag = [&](int r, int c, int s2) __attribute__((always_inline)) {
    uint4 b;
    b.x = relu_bf16x2(pack_bf16(acc[r][c][8 * s2 + 0], acc[r][c][8 * s2 + 1]));
    b.y = relu_bf16x2(pack_bf16(acc[r][c][8 * s2 + 2], acc[r][c][8 * s2 + 3]));
    b.z = relu_bf16x2(pack_bf16(acc[r][c][8 * s2 + 4], acc[r][c][8 * s2 + 5]));
    b.w = relu_bf16x2(pack_bf16(acc[r][c][8 * s2 + 6], acc[r][c][8 * s2 + 7]));
    return b;
  };
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    floatx16 d;
#pragma unroll
    for (int j = 0; j < 16; ++j) d[j] = 0.0f;
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
        d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[r][s2]),
                                                   __builtin_bit_cast(bf16x8, bfrag(r, c, s2)), d, 0, 0, 0);
    dot[c] = d[0];
  }
}

// The first layer over a candidate's own rows: VF_K0_OWN k-steps, steps 0.. of the tile; slot
// n % PD is refilled with step n + PD of the tile.  ONLY: the network has no other hidden
// layer, so these steps are the whole tile - a slot is then refilled with the step that uses it
// next, in this tile or in the next one (possibly the very step it holds: the same fragments
// tile after tile).
template <int RT, int CT, int PD, bool ONLY>
__device__ __forceinline__ void contract_own_rows(floatx16 (&acc)[RT][CT], const floatx16 (&bv)[RT], uint4 (&ring)[PD][RT],
                                                  __amdgpu_buffer_rsrc_t ws, int voff, const uint16_t *bb,
                                                  int cstride) {
  uint4 bcur[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) bcur[c] = *reinterpret_cast<const uint4 *>(bb + (size_t)c * cstride);
  __builtin_amdgcn_s_waitcnt(0x0070);
#pragma unroll
  for (int n = 0; n < VF_K0_OWN; ++n) {
    const int slot = n % PD;
    const int next = (!ONLY || n + PD < VF_K0_OWN) ? n + PD : slot;
#pragma unroll
    for (int i = 0; i < RT * CT; ++i) {
      const int c = i / RT, r = i % RT;
      acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[slot][r]),
                                                         __builtin_bit_cast(bf16x8, bcur[c]), n == 0 ? bv[r] : acc[r][c], 0, 0, 0);
      if (r == RT - 1 && n + 1 < VF_K0_OWN) bcur[c] = *reinterpret_cast<const uint4 *>(bb + (size_t)c * cstride + (n + 1) * 16);
      if (c == CT - 1) ring[slot][r] = stream_load(ws, voff, next * RT + r);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

#endif  // VF_SCORE_DEV_H
