// Device helpers shared by the kernels: storage conversions and the output
// function f of Eq. 1 (branch-specific scale/shift, residual, ReLU, rounding).
#pragma once

#include "cg_internal.h"

namespace cg {

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; NaN stays NaN (gfx950 converts in hardware: v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t float_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

__device__ __forceinline__ float load_as_float(const void* p, long long i, int dtype) {
  return dtype == CG_F32 ? ((const float*)p)[i] : bf16_to_float(((const uint16_t*)p)[i]);
}

// Float paths: s = accumulated sum for the decision taken, fired = d (1 for a dense layer).
__device__ __forceinline__ float finish_float(const Params& p, float s, bool fired, int co, long long o) {
  float a = s;
  if (p.epilogue & CG_EPI_AFFINE) a = fired ? fmaf(p.sc1[co], s, p.sh1[co]) : fmaf(p.sc0[co], s, p.sh0[co]);
  if (p.epilogue & CG_EPI_RESIDUAL) a += load_as_float(p.residual, o, p.out_dtype);
  if (p.epilogue & CG_EPI_RELU) a = fmaxf(a, 0.0f);
  return a;
}

__device__ __forceinline__ void store_float(const Params& p, long long o, float a) {
  if (p.out_dtype == CG_F32)
    ((float*)p.y)[o] = a;
  else
    ((uint16_t*)p.y)[o] = float_to_bf16(a);
}

// Integer path: exact fixed-point requantisation (round half up, arithmetic shift).
__device__ __forceinline__ int32_t finish_int(const Params& p, int32_t s, bool fired, int co, long long o) {
  long long r = 0;
  if (p.epilogue & CG_EPI_RESIDUAL) r = (long long)((const int8_t*)p.residual)[o] * p.rq_res_mult;
  if (p.out_dtype == CG_I32) {
    long long a = (long long)s + r;
    if ((p.epilogue & CG_EPI_RELU) && a < 0) a = 0;
    a = a > 2147483647ll ? 2147483647ll : a;
    a = a < -2147483648ll ? -2147483648ll : a;
    return (int32_t)a;
  }
  long long t = (long long)s * (fired ? p.mult1[co] : p.mult0[co]);
  t += (long long)p.bias[co] * (1ll << p.rq_shift);
  t += r;
  if (p.rq_shift > 0) t = (t + (1ll << (p.rq_shift - 1))) >> p.rq_shift;
  long long lo = (p.epilogue & CG_EPI_RELU) ? 0 : -128;
  t = t < lo ? lo : t;
  t = t > 127 ? 127 : t;
  return (int32_t)t;
}

__device__ __forceinline__ void store_int(const Params& p, long long o, int32_t v) {
  if (p.out_dtype == CG_I32)
    ((int32_t*)p.y)[o] = v;
  else
    ((int8_t*)p.y)[o] = (int8_t)v;
}

}  // namespace cg
