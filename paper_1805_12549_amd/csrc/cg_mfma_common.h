// Pieces shared by the matrix-core kernels: vector types, the bf16 / int8 MFMA traits and
// the whole-row output function (f of Eq. 1 applied to eight consecutive channels).
#pragma once

#include "cg_device.h"

namespace cg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

struct Bf16Traits {
  using acc4 = f32x4;
  using acc_t = float;
  static constexpr int kDtype = CG_BF16;
  // 16x16 output block, K = 32: lane l supplies row/column l%16 and the 8 elements
  // (one 16-byte chunk) number l/16 of the K slice, for A and B alike.
  static __device__ __forceinline__ acc4 mfma(i32x4 a, i32x4 b, acc4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
  static __device__ __forceinline__ bool fires(float v, float lo, float hi) { return v >= lo && v <= hi; }
};

struct I8Traits {
  using acc4 = i32x4;
  using acc_t = int32_t;
  static constexpr int kDtype = CG_I8;
  static __device__ __forceinline__ acc4 mfma(i32x4 a, i32x4 b, acc4 c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ bool fires(int32_t v, int32_t lo, int32_t) { return v >= lo; }
};

__device__ __forceinline__ int shfl_xor_i(int v, int mask) { return __shfl_xor(v, mask, 64); }

// Output function for eight consecutive channels co0..co0+7 of one output pixel, into registers.
// s0, s1: the eight sums (fp32 bit patterns or int32); dbyte: their decisions, bit k = channel co0+k;
// o: element offset of channel co0 in y / residual.  The converted values come back packed in
// out0 (and out1 for 4-byte outputs): 32 bytes for CG_F32 / CG_I32, 16 for CG_BF16, 8 for CG_I8.
template <typename Tr>
__device__ __forceinline__ void finish8(const Params& p, i32x4 s0, i32x4 s1, uint32_t dbyte, int co0, long long o,
                                        i32x4& out0, i32x4& out1) {
  out0 = i32x4{0, 0, 0, 0};
  out1 = i32x4{0, 0, 0, 0};
  if constexpr (Tr::kDtype == CG_I8) {
    int32_t v[8];
    int8_t res8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (p.epilogue & CG_EPI_RESIDUAL) *(uint2*)res8 = *(const uint2*)((const int8_t*)p.residual + o);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int32_t s = k < 4 ? s0[k] : s1[k - 4];
      const bool f = p.gated ? ((dbyte >> k) & 1u) : true;
      const int co = co0 + k;
      const long long r = (p.epilogue & CG_EPI_RESIDUAL) ? (long long)res8[k] * p.rq_res_mult : 0;
      if (p.out_dtype == CG_I32) {
        long long a = (long long)s + r;
        if ((p.epilogue & CG_EPI_RELU) && a < 0) a = 0;
        a = a > 2147483647ll ? 2147483647ll : a;
        a = a < -2147483648ll ? -2147483648ll : a;
        v[k] = (int32_t)a;
      } else {
        long long t = (long long)s * (f ? p.mult1[co] : p.mult0[co]);
        t += (long long)p.bias[co] * (1ll << p.rq_shift);
        t += r;
        if (p.rq_shift > 0) t = (t + (1ll << (p.rq_shift - 1))) >> p.rq_shift;
        const long long lo = (p.epilogue & CG_EPI_RELU) ? 0 : -128;
        t = t < lo ? lo : t;
        t = t > 127 ? 127 : t;
        v[k] = (int32_t)t;
      }
    }
    if (p.out_dtype == CG_I32) {
      out0 = i32x4{v[0], v[1], v[2], v[3]};
      out1 = i32x4{v[4], v[5], v[6], v[7]};
    } else {
      out0[0] = (v[0] & 0xff) | ((v[1] & 0xff) << 8) | ((v[2] & 0xff) << 16) | ((v[3] & 0xff) << 24);
      out0[1] = (v[4] & 0xff) | ((v[5] & 0xff) << 8) | ((v[6] & 0xff) << 16) | ((v[7] & 0xff) << 24);
    }
  } else {
    float v[8];
    float res[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (p.epilogue & CG_EPI_RESIDUAL) {
      if (p.out_dtype == CG_F32) {
        const f32x4 r0 = *(const f32x4*)((const float*)p.residual + o);
        const f32x4 r1 = *(const f32x4*)((const float*)p.residual + o + 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          res[k] = r0[k];
          res[k + 4] = r1[k];
        }
      } else {
        uint16_t rb[8];
        *(i32x4*)rb = *(const i32x4*)((const uint16_t*)p.residual + o);
#pragma unroll
        for (int k = 0; k < 8; ++k) res[k] = bf16_to_float(rb[k]);
      }
    }
    // the two scale/shift pairs of the eight channels as 16-byte loads (co0 is a multiple of 8)
    float sc0[8], sh0[8], sc1[8], sh1[8];
    if (p.epilogue & CG_EPI_AFFINE) {
#pragma unroll
      for (int h4 = 0; h4 < 2; ++h4) {
        const f32x4 a0 = *(const f32x4*)(p.sc0 + co0 + 4 * h4), b0 = *(const f32x4*)(p.sh0 + co0 + 4 * h4);
        const f32x4 a1 = *(const f32x4*)(p.sc1 + co0 + 4 * h4), b1 = *(const f32x4*)(p.sh1 + co0 + 4 * h4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sc0[4 * h4 + e] = a0[e];
          sh0[4 * h4 + e] = b0[e];
          sc1[4 * h4 + e] = a1[e];
          sh1[4 * h4 + e] = b1[e];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float s = __int_as_float(k < 4 ? s0[k] : s1[k - 4]);
      const bool f = p.gated ? ((dbyte >> k) & 1u) : true;
      float a = s;
      if (p.epilogue & CG_EPI_AFFINE) a = f ? fmaf(sc1[k], s, sh1[k]) : fmaf(sc0[k], s, sh0[k]);
      if (p.epilogue & CG_EPI_RESIDUAL) a += res[k];
      if (p.epilogue & CG_EPI_RELU) a = fmaxf(a, 0.0f);
      v[k] = a;
    }
    if (p.out_dtype == CG_F32) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        out0[k] = __float_as_int(v[k]);
        out1[k] = __float_as_int(v[k + 4]);
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        out0[k] = (int)((uint32_t)float_to_bf16(v[2 * k]) | ((uint32_t)float_to_bf16(v[2 * k + 1]) << 16));
    }
  }
}

// the same, stored to y
template <typename Tr>
__device__ __forceinline__ void finish_store8(const Params& p, i32x4 s0, i32x4 s1, uint32_t dbyte, int co0,
                                              long long o) {
  i32x4 a, b;
  finish8<Tr>(p, s0, s1, dbyte, co0, o, a, b);
  if (p.out_dtype == CG_F32 || p.out_dtype == CG_I32) {
    *(i32x4*)((int32_t*)p.y + o) = a;
    *(i32x4*)((int32_t*)p.y + o + 4) = b;
  } else if (p.out_dtype == CG_BF16) {
    *(i32x4*)((uint16_t*)p.y + o) = a;
  } else {
    *(int2*)((int8_t*)p.y + o) = int2{a[0], a[1]};
  }
}

}  // namespace cg
