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

// (value, id) ordering of the scan: smaller value first, then smaller id; id < 0 = none
__device__ __forceinline__ void take_min(float &v, int32_t &c, float ov, int32_t oc) {
  if (oc >= 0 && (ov < v || (ov == v && (c < 0 || oc < c)))) { v = ov; c = oc; }
}
__device__ __forceinline__ void wave_min(float &v, int32_t &c) {
  for (int off = 32; off > 0; off >>= 1) {
    float ov = __shfl_down(v, off);
    int32_t oc = __shfl_down(c, off);
    take_min(v, c, ov, oc);
  }
}

// gate non-linearities of the recurrent network, fp32
__device__ __forceinline__ float sigmoid_dev(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float tanh_dev(float z) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * z)); }

#endif  // VF_SCORE_DEV_H
