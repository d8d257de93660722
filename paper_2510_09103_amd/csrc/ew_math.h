// Element-wise arithmetic shared by the streaming kernels, written for a small instruction
// count per element: the update is memory-bound only if it stays well under ~40 vector
// instructions per element on gfx950.
//   u  = clip( m^c * inv ),   inv = 1 / (sqrt(v) + eps)        (Alg. 1 last line)
//   W' = W (1 - lr lambda) - lr u                              (the same line, regrouped)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adapm {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2_t v = {a, b};
  bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&h);
}

// (x0, x1) -> packed hi = bf16(x), packed lo = bf16(x - hi)
__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16x2(x0, x1);
  lo = pack_bf16x2(x0 - bf16lo(hi), x1 - bf16hi(hi));
}

// sum of squares of two packed bf16 values added to acc (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_sq(uint32_t w, float acc) {
  bf16x2_t a = *reinterpret_cast<bf16x2_t*>(&w);
  return __builtin_amdgcn_fdot2_f32_bf16(a, a, acc, false);
}

// 1 / (sqrt(v * idv) + eps) * idm with the hardware sqrt / rcp (about 1 ulp each)
__device__ __forceinline__ float inv_denom_fast(float v, float idv, float idm, float eps) {
  return idm * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v * idv) + eps);
}
// the same with correctly rounded sqrt and divide (used once per group of rows)
__device__ __forceinline__ float inv_denom_exact(float v, float idv, float idm, float eps) {
  return idm / (sqrtf(v * idv) + eps);
}

struct UpdCoef {
  float neg_lrs;   // -lr * lr_scale
  float decay;     // 1 - lr * lr_scale * lambda
  float clip;
};

__device__ __forceinline__ UpdCoef make_coef(float lr, float lr_scale, float wd, float clip) {
  UpdCoef c;
  const float lrs = lr * lr_scale;
  c.neg_lrs = -lrs;
  c.decay = 1.f - lrs * wd;
  c.clip = clip;
  return c;
}

__device__ __forceinline__ float apply_update(float w, float mc, float inv, const UpdCoef& c) {
  const float u = __builtin_amdgcn_fmed3f(mc * inv, -c.clip, c.clip);
  return fmaf(c.neg_lrs, u, w * c.decay);
}

// The same with the factor -lr folded into the per-row inverse: ninv = -lr * inv, bound = lr * clip.
// Three instructions per element (multiply, median, fused multiply-add).
__device__ __forceinline__ float apply_update_scaled(float w, float mc, float ninv, float bound, float decay) {
  return fmaf(w, decay, __builtin_amdgcn_fmed3f(mc * ninv, -bound, bound));
}

}  // namespace adapm
