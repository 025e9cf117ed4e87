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

// gate non-linearities of the recurrent network, fp32
__device__ __forceinline__ float sigmoid_dev(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float tanh_dev(float z) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * z)); }

#endif  // VF_SCORE_DEV_H
