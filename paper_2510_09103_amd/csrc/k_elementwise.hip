// Streaming kernels of the AdaPM step: blockwise second-moment statistics,
// the fused element-wise update, state initialisation.
//
//  - v statistics: v_g <- beta2 v_g + (1-beta2) mean_{i in g} G_i^2 (Alg. 1 "v_t" with the
//    blockwise mean of Sec. 5.1.3).  A group is a contiguous run of elements (whole rows),
//    reduced by one wavefront with DPP-style shuffles; long groups go through fixed-order
//    partial sums (deterministic, no float atomics).
//  - update: m <- (1-beta1) G + beta1 m (eq. 5) or m^c = cG G + cC C for low-rank blocks
//    (eq. 4 rewritten as m^c = G + beta1/(1-beta1) (L_{t-1}R_{t-1} - L_t R_t)), per-element v,
//    then W <- W - lr (clip(m^c / (sqrt(v) + eps)) + lambda W)  (Alg. 1 last line).
#include "adapm_plan.h"
#include "ew_math.h"

namespace adapm {

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void load8(const char* base, int dtype, int64_t e, float out[8]) {
  if (dtype == DT_BF16) {
    uint4 q = *reinterpret_cast<const uint4*>(base + e * 2);
    uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
    float4 a = *reinterpret_cast<const float4*>(base + e * 4);
    float4 b = *reinterpret_cast<const float4*>(base + e * 4 + 16);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
  }
}

__device__ __forceinline__ void store8(char* base, int dtype, int64_t e, const float in[8]) {
  if (dtype == DT_BF16) {
    *reinterpret_cast<uint4*>(base + e * 2) = make_uint4(pack_bf16x2(in[0], in[1]), pack_bf16x2(in[2], in[3]),
                                                         pack_bf16x2(in[4], in[5]), pack_bf16x2(in[6], in[7]));
  } else {
    *reinterpret_cast<float4*>(base + e * 4) = make_float4(in[0], in[1], in[2], in[3]);
    *reinterpret_cast<float4*>(base + e * 4 + 16) = make_float4(in[4], in[5], in[6], in[7]);
  }
}

__device__ __forceinline__ float load1(const char* base, int dtype, int64_t e) {
  return dtype == DT_BF16 ? bf16_to_f32(*reinterpret_cast<const uint16_t*>(base + e * 2))
                          : *reinterpret_cast<const float*>(base + e * 4);
}

__device__ __forceinline__ void store1(char* base, int dtype, int64_t e, float x) {
  if (dtype == DT_BF16) *reinterpret_cast<uint16_t*>(base + e * 2) = f32_to_bf16_rne(x);
  else *reinterpret_cast<float*>(base + e * 4) = x;
}

// ---------------------------------------------------------------------------
// v statistics
// ---------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

__global__ __launch_bounds__(256) void vstat_kernel(const BlockDev* __restrict__ blocks,
                                                    const VsItem* __restrict__ items, int64_t nitems,
                                                    double* __restrict__ partials, Bases b, float beta2) {
  const int lane = threadIdx.x & 63;
  const int64_t it = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (it >= nitems) return;
  const VsItem item = items[it];
  const BlockDev blk = blocks[item.block];
  const char* G = (const char*)b.grads[item.block];
  const int64_t s = item.start, e = item.start + item.count;
  const int64_t a0 = min((s + 7) & ~(int64_t)7, e), a1 = max(e & ~(int64_t)7, a0);
  float acc = 0.f;
  for (int64_t i = s + lane; i < a0; i += 64) { float g = load1(G, blk.grad_dtype, i); acc += g * g; }
  if (blk.grad_dtype == DT_BF16) {
    for (int64_t i = a0 + (int64_t)lane * 8; i < a1; i += 512) {
      const uint4 q = *reinterpret_cast<const uint4*>(G + i * 2);
      acc += dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
    }
  } else {
    for (int64_t i = a0 + (int64_t)lane * 8; i < a1; i += 512) {
      float g[8];
      load8(G, DT_F32, i, g);
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) t += g[k] * g[k];
      acc += t;
    }
  }
  for (int64_t i = a1 + lane; i < e; i += 64) { float g = load1(G, blk.grad_dtype, i); acc += g * g; }
  const float gs = grad_scale(b);                 // global clipping: the method sees gs * G
  double sum = wave_sum((double)acc) * ((double)gs * (double)gs);
  if (lane == 0) {
    if (item.direct) {
      float* v = reinterpret_cast<float*>(b.state + blk.off_v) + item.out;
      *v = (float)((double)beta2 * (double)*v + (1.0 - (double)beta2) * (sum / (double)blk.group_elems));
    } else {
      partials[item.out] = sum;
    }
  }
}

__global__ __launch_bounds__(256) void vfinal_kernel(const BlockDev* __restrict__ blocks,
                                                     const VfItem* __restrict__ items, int64_t nitems,
                                                     const double* __restrict__ partials, Bases b, float beta2) {
  const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (it >= nitems) return;
  const VfItem item = items[it];
  const BlockDev blk = blocks[item.block];
  double sum = 0.0;
  for (int p = 0; p < item.nparts; ++p) sum += partials[item.part0 + p];
  float* v = reinterpret_cast<float*>(b.state + blk.off_v) + item.group;
  *v = (float)((double)beta2 * (double)*v + (1.0 - (double)beta2) * (sum / (double)blk.group_elems));
}

// Global gradient-norm clipping: partial sums of squares of every gradient (made by vstat_kernel, one per
// piece, no scaling) -> norm and factor, summed in a fixed order.  out[0] = norm, out[1] = factor.
__global__ __launch_bounds__(1024) void gradnorm_final_kernel(const double* __restrict__ partials, int64_t nparts,
                                                              float max_norm, float* __restrict__ out) {
  __shared__ double red[1024];
  double s = 0.0;
  for (int64_t i = threadIdx.x; i < nparts; i += 1024) s += partials[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double norm = sqrt(red[0]);
    const double f = (double)max_norm / (norm + 1e-6);
    out[0] = (float)norm;
    out[1] = (float)(f < 1.0 ? f : 1.0);
  }
}

// Full / no momentum blocks with a blockwise second moment whose groups fit a wavefront's registers
// (bf16 G and W, at most GRP_MAX_ELEMS elements, a multiple of 8: e.g. one v per 1600-element row of an embedding):
// statistic and update in one pass.  A wave reads its group of G once, reduces sum G^2 (fp32 per lane, fp64
// across lanes, the same arithmetic as vstat_kernel), updates v_g and then W (and m) with G still in registers.
__global__ __launch_bounds__(256) void update_grouped_kernel(const BlockDev* __restrict__ blocks,
                                                             const GrpItem* __restrict__ items, Bases b, StepScalars sc) {
  const GrpItem item = items[blockIdx.x];
  const BlockDev blk = blocks[item.block];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const char* G = (const char*)b.grads[item.block];
  char* W = (char*)b.params[item.block];
  float* m = blk.off_m >= 0 ? reinterpret_cast<float*>(b.state + blk.off_m) : nullptr;
  float* v = reinterpret_cast<float*>(b.state + blk.off_v);
  const UpdCoef cf = make_coef(sc.lr, blk.lr_scale, blk.wd, sc.clip);
  const float ob1 = 1.f - sc.beta1;
  const float gs = grad_scale(b);                 // global clipping: the method sees gs * G
  const int ge = (int)blk.group_elems, nvec = ge >> 3;
  for (int64_t g = item.g0 + wave; g < item.g0 + item.ngroups; g += 4) {
    const int64_t base = g * ge;
    // G, W and m of the whole group are requested together, as raw vectors on clamped (always valid) indices, and
    // converted afterwards (W and m do not depend on v): one memory latency per group.  bf16 G and W only.
    uint4 gq[4], wq[4];
    float4 ma[4], mb[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int iv = lane + 64 * k;
      const int64_t e0 = base + (int64_t)(iv < nvec ? iv : nvec - 1) * 8;
      gq[k] = *reinterpret_cast<const uint4*>(G + e0 * 2);
      wq[k] = *reinterpret_cast<const uint4*>(W + e0 * 2);
      if (m) {
        ma[k] = *reinterpret_cast<const float4*>(m + e0);
        mb[k] = *reinterpret_cast<const float4*>(m + e0 + 4);
      }
    }
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (lane + 64 * k < nvec) acc += dot2_sq(gq[k].w, dot2_sq(gq[k].z, dot2_sq(gq[k].y, dot2_sq(gq[k].x, 0.f))));
    const double sum = wave_sum((double)acc) * ((double)gs * (double)gs);
    const float vn = (float)((double)sc.beta2 * (double)v[g] + (1.0 - (double)sc.beta2) * (sum / (double)ge));
    if (lane == 0) v[g] = vn;
    const float inv = inv_denom_exact(vn, sc.inv_debias_v, sc.inv_debias_m, sc.eps);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int iv = lane + 64 * k;
      if (iv < nvec) {
        const int64_t e0 = base + (int64_t)iv * 8;
        const uint32_t gw[4] = {gq[k].x, gq[k].y, gq[k].z, gq[k].w}, ww[4] = {wq[k].x, wq[k].y, wq[k].z, wq[k].w};
        float mc[8], w[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          mc[2 * e] = gs * __uint_as_float(gw[e] << 16);
          mc[2 * e + 1] = gs * __uint_as_float(gw[e] & 0xffff0000u);
          w[2 * e] = __uint_as_float(ww[e] << 16);
          w[2 * e + 1] = __uint_as_float(ww[e] & 0xffff0000u);
        }
        if (m) {                                  // full momentum, eq. 5
          const float mo[8] = {ma[k].x, ma[k].y, ma[k].z, ma[k].w, mb[k].x, mb[k].y, mb[k].z, mb[k].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) mc[e] = ob1 * mc[e] + sc.beta1 * mo[e];
          store8((char*)m, DT_F32, e0, mc);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = apply_update(w[e], mc[e], inv, cf);
        store8(W, DT_BF16, e0, w);
      }
    }
  }
}

// Normaliser of the optional scale-normalised Alg. 2: s = 1 / max(||R R^T||_F, ||L^T L||_F) from the two Gram
// matrices of the iteration (fp64 sums in a fixed order).
__global__ __launch_bounds__(256) void gram_norm_kernel(const GnormItem* __restrict__ items, Bases b) {
  __shared__ double red[2][256];
  const GnormItem it = items[blockIdx.x];
  const int n = it.r * it.r;
  double sa = 0.0, sb = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) {
    double x, y;
    if (it.dtype == DT_F64) {
      x = reinterpret_cast<const double*>(b.ws + it.off_a)[i];
      y = reinterpret_cast<const double*>(b.ws + it.off_b)[i];
    } else {
      x = (double)reinterpret_cast<const float*>(b.ws + it.off_a)[i];
      y = (double)reinterpret_cast<const float*>(b.ws + it.off_b)[i];
    }
    sa += x * x;
    sb += y * y;
  }
  red[0][threadIdx.x] = sa;
  red[1][threadIdx.x] = sb;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) { red[0][threadIdx.x] += red[0][threadIdx.x + w]; red[1][threadIdx.x] += red[1][threadIdx.x + w]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nu = sqrt(red[0][0] > red[1][0] ? red[0][0] : red[1][0]);
    *reinterpret_cast<double*>(b.ws + it.off_out) = nu > 0.0 ? 1.0 / nu : 1.0;
  }
}

// ---------------------------------------------------------------------------
// fused update
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void update_kernel(const BlockDev* __restrict__ blocks,
                                                     const EwItem* __restrict__ items, Bases b, StepScalars sc) {
  const EwItem item = items[blockIdx.x];
  const BlockDev blk = blocks[item.block];
  const char* G = (const char*)b.grads[item.block];
  char* W = (char*)b.params[item.block];
  float* m = blk.off_m >= 0 ? reinterpret_cast<float*>(b.state + blk.off_m) : nullptr;
  float* v = reinterpret_cast<float*>(b.state + blk.off_v);
  const float* C = blk.off_C >= 0 ? reinterpret_cast<const float*>(b.ws + blk.off_C) : nullptr;
  const UpdCoef cf = make_coef(sc.lr, blk.lr_scale, blk.wd, sc.clip);
  const float ob1 = 1.f - sc.beta1, ob2 = 1.f - sc.beta2;
  const float gs = grad_scale(b);                 // global clipping: the method sees gs * G
  const int nvec = (item.count + 7) >> 3;
  const int64_t end = item.start + item.count;
  // group index of this thread's first vector; later vectors advance by 2048 elements
  const int64_t ge = blk.group_elems;
  int64_t grp = 0, rem = 0, dq = 0, dr = 0;
  if (blk.v_mode != VM_ELEMENT) {
    const int64_t e0 = item.start + (int64_t)threadIdx.x * 8;
    if (ge < (1ll << 31) && e0 < (1ll << 31)) { grp = (uint32_t)e0 / (uint32_t)ge; rem = (uint32_t)e0 % (uint32_t)ge; dq = 2048u / (uint32_t)ge; dr = 2048u % (uint32_t)ge; }
    else { grp = e0 / ge; rem = e0 % ge; dq = 2048 / ge; dr = 2048 % ge; }
  }
  for (int iv = threadIdx.x; iv < nvec; iv += 256) {
    const int64_t e = item.start + (int64_t)iv * 8;
    if (e + 8 <= end) {
      float g[8], w[8], inv[8], mc[8];
      load8(G, blk.grad_dtype, e, g);
      if (gs != 1.f) {
#pragma unroll
        for (int k = 0; k < 8; ++k) g[k] *= gs;
      }
      load8(W, blk.param_dtype, e, w);
      if (blk.v_mode == VM_ELEMENT) {
        float vv[8];
        load8((const char*)v, DT_F32, e, vv);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          vv[k] = sc.beta2 * vv[k] + ob2 * g[k] * g[k];
          inv[k] = inv_denom_fast(vv[k], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
        }
        store8((char*)v, DT_F32, e, vv);
      } else if (rem + 8 <= ge) {
        const float x = inv_denom_fast(v[grp], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
#pragma unroll
        for (int k = 0; k < 8; ++k) inv[k] = x;
      } else {
        int64_t gk = grp, rk = rem;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          inv[k] = inv_denom_fast(v[gk], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
          if (++rk == ge) { rk = 0; ++gk; }
        }
      }
      if (blk.mom_mode == MM_FULL) {            // full momentum, eq. 5
        load8((const char*)m, DT_F32, e, mc);
#pragma unroll
        for (int k = 0; k < 8; ++k) mc[k] = ob1 * g[k] + sc.beta1 * mc[k];
        store8((char*)m, DT_F32, e, mc);
      } else if (blk.mom_mode == MM_LOWRANK) {  // low-rank: m^c = cG G + cC C
        load8((const char*)C, DT_F32, e, mc);
#pragma unroll
        for (int k = 0; k < 8; ++k) mc[k] = sc.cG * g[k] + sc.cC * mc[k];
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) mc[k] = g[k];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) w[k] = apply_update(w[k], mc[k], inv[k], cf);
      store8(W, blk.param_dtype, e, w);
    } else {
      int64_t gk = grp, rk = rem;
      for (int64_t i = e; i < end; ++i) {
        const float g = load1(G, blk.grad_dtype, i) * gs;
        const float w = load1(W, blk.param_dtype, i);
        float vv;
        if (blk.v_mode == VM_ELEMENT) {
          vv = sc.beta2 * v[i] + ob2 * g * g;
          v[i] = vv;
        } else {
          vv = v[gk];
          if (++rk == ge) { rk = 0; ++gk; }
        }
        float mc;
        if (blk.mom_mode == MM_FULL) { mc = ob1 * g + sc.beta1 * m[i]; m[i] = mc; }
        else if (blk.mom_mode == MM_LOWRANK) mc = sc.cG * g + sc.cC * C[i];
        else mc = g;
        store1(W, blk.param_dtype, i,
               apply_update(w, mc, inv_denom_fast(vv, sc.inv_debias_v, sc.inv_debias_m, sc.eps), cf));
      }
    }
    if (blk.v_mode != VM_ELEMENT) {
      grp += dq; rem += dr;
      if (rem >= ge) { rem -= ge; ++grp; }
    }
  }
}

// ---------------------------------------------------------------------------
// state initialisation
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
    p[i] = make_uint4(0, 0, 0, 0);
}

// plain copy of fp32 arrays (the factors of Alg. 2 into the state where nothing else has to be done to them)
__global__ __launch_bounds__(256) void copy_kernel(const CopyItem* __restrict__ items, Bases bs) {
  const CopyItem it = items[blockIdx.x];
  const float* __restrict__ src = reinterpret_cast<const float*>(resolve(it.src, bs)) + it.first;
  float* __restrict__ dst = reinterpret_cast<float*>(resolve(it.dst, bs)) + it.first;
  const int n4 = it.count >> 2;
  for (int i = threadIdx.x; i < n4; i += 256)
    reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
  for (int i = 4 * n4 + threadIdx.x; i < it.count; i += 256) dst[i] = src[i];
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {   // SplitMix64 finaliser
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// R_0[i] = fp32(k_i) * amp,  k_i = (mix64(key + i) >> 40) - 2^23: a counter-based uniform sketch.
__global__ __launch_bounds__(256) void sketch_kernel(const SketchItem* __restrict__ items, char* state) {
  const SketchItem it = items[blockIdx.y];
  float* R = reinterpret_cast<float*>(state + it.off_R);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < it.count; i += (int64_t)gridDim.x * 256) {
    const int32_t k = (int32_t)(mix64(it.key + (uint64_t)i) >> 40) - (1 << 23);
    R[i] = __fmul_rn((float)k, it.amp);
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
void launch_vstat(const BlockDev* blocks, const VsItem* items, int64_t nitems, double* partials, Bases b,
                  float beta2, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(vstat_kernel, dim3((unsigned)((nitems + 3) / 4)), dim3(256), 0, s, blocks, items, nitems,
                     partials, b, beta2);
}

void launch_vfinal(const BlockDev* blocks, const VfItem* items, int64_t nitems, const double* partials, Bases b,
                   float beta2, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(vfinal_kernel, dim3((unsigned)((nitems + 255) / 256)), dim3(256), 0, s, blocks, items, nitems,
                     partials, b, beta2);
}

void launch_update_grouped(const BlockDev* blocks, const GrpItem* items, int64_t nitems, Bases b, StepScalars sc,
                           hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(update_grouped_kernel, dim3((unsigned)nitems), dim3(256), 0, s, blocks, items, b, sc);
}

void launch_gram_norm(const GnormItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(gram_norm_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

void launch_gradnorm_final(const double* partials, int64_t nparts, float max_norm, float* out, hipStream_t s) {
  hipLaunchKernelGGL(gradnorm_final_kernel, dim3(1), dim3(1024), 0, s, partials, nparts, max_norm, out);
}

void launch_update(const BlockDev* blocks, const EwItem* items, int64_t nitems, Bases b, StepScalars sc,
                   hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(update_kernel, dim3((unsigned)nitems), dim3(256), 0, s, blocks, items, b, sc);
}

void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return;
  const int64_t n16 = (int64_t)(bytes / 16);
  const unsigned grid = (unsigned)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<uint4*>(p), n16);
}

void launch_copy(const CopyItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

void launch_sketch(const SketchItem* items, int64_t nitems, char* state, hipStream_t s) {
  if (nitems <= 0) return;
  for (int64_t i0 = 0; i0 < nitems; i0 += 32768) {
    const unsigned ny = (unsigned)(nitems - i0 < 32768 ? nitems - i0 : 32768);
    hipLaunchKernelGGL(sketch_kernel, dim3(64, ny), dim3(256), 0, s, items + i0, state);
  }
}

}  // namespace adapm
