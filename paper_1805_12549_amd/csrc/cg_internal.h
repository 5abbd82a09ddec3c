// Internal declarations shared by the host API and the kernels of the
// channel-gated convolution library.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cg_conv.h"

namespace cg {

// Everything a kernel needs to know about one forward call; passed by value.
struct Params {
  int n, h, w, c_in, c_out, c_base, c_cond;
  int kh, kw, stride, pad, ho, wo;
  long long x_pixel_stride;
  long long m_total;       // n*ho*wo
  unsigned epilogue;
  int in_dtype, out_dtype;
  int gated;               // 0: dense layer, no gate, second affine pair applies
  int rq_shift, rq_res_mult;
  int words;               // bitmap words per pixel = ceil(c_out/32)

  // per-output-channel tables, device, in `packed`
  const float* thr_f;      // lower threshold on the fp32 base sum (Sec. 3.2 merged gate)
  const float* thr_hi_f;   // upper threshold (+inf when one-sided)
  const int32_t* thr_i;    // integer threshold (int8 path)
  const float *sc0, *sh0, *sc1, *sh1;
  const int32_t *mult0, *mult1, *bias;

  // weights in caller layout [c_out][kh][kw][c], copied into `packed`
  const void* w_base;
  const void* w_cond;

  // call arguments
  const void* x;
  const void* residual;
  void* y;
  uint32_t* bitmap;
  uint32_t* counts;
};

// Repacked-weight geometry of the matrix-core kernels (filled by mfma_plan).
struct MfmaPlan {
  int ok;                // 0: shape not supported by the matrix-core kernels
  int elem_bytes;        // 2 (bf16) or 1 (int8)
  int chunk;             // channels per 16-byte chunk: 8 (bf16) or 16 (int8)
  int bm, bn;            // workgroup tile: output pixels x output channels
  int kq_base, kq_cond;  // K extent in 16-byte chunks, padded to a multiple of 4 (one MFMA step)
  size_t wpk_base_bytes, wpk_cond_bytes;
};

MfmaPlan mfma_plan(const cg_conv_desc& d);

// launchers (return hipError_t from the last launch)
hipError_t launch_naive(const Params& p, hipStream_t s);
hipError_t launch_zero_u32(uint32_t* ptr, size_t words, hipStream_t s);
hipError_t launch_mfma_pack(const MfmaPlan& plan, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s);
hipError_t launch_mfma(const MfmaPlan& plan, const Params& p, const void* wpk_base, const void* wpk_cond,
                       hipStream_t s);

}  // namespace cg
