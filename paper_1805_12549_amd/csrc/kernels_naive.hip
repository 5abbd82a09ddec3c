// Plain kernel: one thread per output activation, direct convolution.
// Covers every shape and dtype the API accepts (fp32 layers, channel counts
// the matrix-core kernels cannot tile, any kernel size).  Follows Eq. 1 of
// the channel-gating paper step by step: base sum, gate, conditional sum only
// where the gate fired, output function.  With channel grouping (Sec. 3.3) the
// base channels of output group i are input group i and the conditional
// channels are all the others in increasing order.
#include "cg_device.h"

namespace cg {

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  using acc_t = float;
  static __device__ __forceinline__ float mul_add(float a, float b, float c) { return fmaf(a, b, c); }
  static __device__ __forceinline__ float get(const float* p, long long i) { return p[i]; }
};
template <>
struct Elem<uint16_t> {
  using acc_t = float;
  static __device__ __forceinline__ float mul_add(float a, float b, float c) { return fmaf(a, b, c); }
  static __device__ __forceinline__ float get(const uint16_t* p, long long i) { return bf16_to_float(p[i]); }
};
template <>
struct Elem<int8_t> {
  using acc_t = int32_t;
  static __device__ __forceinline__ int32_t mul_add(int32_t a, int32_t b, int32_t c) { return a * b + c; }
  static __device__ __forceinline__ int32_t get(const int8_t* p, long long i) { return p[i]; }
};

// Thread t handles activation (m, co) with t = m * (32*words) + co: every 32-lane half
// of a wavefront is exactly one bitmap word, so the ballot mask is the word.
template <typename T>
__global__ __launch_bounds__(256) void naive_kernel(Params p) {
  using E = Elem<T>;
  using acc_t = typename E::acc_t;
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int cpad = p.words * 32;
  const long long m = t / cpad;
  const int co = (int)(t - m * cpad);
  const bool live = m < p.m_total && co < p.c_out;

  bool fired = false;
  if (live) {
    const int wo = (int)(m % p.wo);
    const long long q = m / p.wo;
    const int ho = (int)(q % p.ho);
    const int img = (int)(q / p.ho);
    const T* x = (const T*)p.x;
    const T* wb = (const T*)p.w_base + (long long)co * p.kh * p.kw * p.c_base;
    const T* wc = (const T*)p.w_cond + (long long)co * p.kh * p.kw * p.c_cond;

    const int grp = co / p.cpg;           // 0 without grouping
    const int b0 = grp * p.c_base;        // first base-path channel of this output channel

    acc_t acc = 0;
    for (int r = 0; r < p.kh; ++r) {
      const int hi = ho * p.stride - p.pad + r;
      if (hi < 0 || hi >= p.h) continue;
      for (int s = 0; s < p.kw; ++s) {
        const int wi = wo * p.stride - p.pad + s;
        if (wi < 0 || wi >= p.w) continue;
        const long long xo = (((long long)img * p.h + hi) * p.w + wi) * p.x_pixel_stride;
        const int wofs = (r * p.kw + s) * p.c_base;
        for (int c = 0; c < p.c_base; ++c) acc = E::mul_add(E::get(x, xo + b0 + c), E::get(wb, wofs + c), acc);
      }
    }

    if (p.gated) {
      if constexpr (__is_same(acc_t, int32_t)) {
        fired = acc >= p.thr_i[co];
      } else {
        fired = (acc >= p.thr_f[co]) && (acc <= p.thr_hi_f[co]);
      }
      if (p.chan_mask) fired = fired && ((p.chan_mask[(long long)img * p.words + (co >> 5)] >> (co & 31)) & 1u);
      if (fired && !p.gate_only) {
        for (int r = 0; r < p.kh; ++r) {
          const int hi = ho * p.stride - p.pad + r;
          if (hi < 0 || hi >= p.h) continue;
          for (int s = 0; s < p.kw; ++s) {
            const int wi = wo * p.stride - p.pad + s;
            if (wi < 0 || wi >= p.w) continue;
            const long long xo = (((long long)img * p.h + hi) * p.w + wi) * p.x_pixel_stride;
            const int wofs = (r * p.kw + s) * p.c_cond;
            // conditional channel c is input channel c below the base channels, c + c_base above
            for (int c = 0; c < b0; ++c) acc = E::mul_add(E::get(x, xo + c), E::get(wc, wofs + c), acc);
            for (int c = b0; c < p.c_cond; ++c)
              acc = E::mul_add(E::get(x, xo + p.c_base + c), E::get(wc, wofs + c), acc);
          }
        }
      }
    }

    if (!p.gate_only) {
      const long long o = m * p.c_out + (p.shuffle ? (co - grp * p.cpg) * p.groups + grp : co);
      const bool branch1 = p.gated ? fired : true;
      if constexpr (__is_same(acc_t, float)) {
        store_float(p, o, finish_float(p, acc, branch1, co, o));
      } else {
        store_int(p, o, finish_int(p, acc, branch1, co, o));
      }
    }
    if (fired && p.counts) atomicAdd(&p.counts[2 + (long long)img * p.c_out + co], 1u);
  }

  const unsigned long long mask = __ballot(fired);
  const int lane = threadIdx.x & 63;
  if (p.bitmap && (lane & 31) == 0 && m < p.m_total)
    p.bitmap[t >> 5] = (uint32_t)(lane ? (mask >> 32) : mask);
  if (p.counts && lane == 0 && mask) {
    atomicAdd((unsigned long long*)p.counts, (unsigned long long)__popcll(mask));
  }
}

__global__ void zero_u32_kernel(uint32_t* ptr, size_t words) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < words) ptr[i] = 0u;
}

__global__ void chan_mask_kernel(const uint32_t* __restrict__ counts, int n, int c_out, int words, uint32_t need,
                                 uint32_t* __restrict__ mask) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n * words) return;
  const int img = i / words, w = i - img * words;
  uint32_t bits = 0u;
  for (int b = 0; b < 32; ++b) {
    const int co = 32 * w + b;
    if (co < c_out && counts[2 + (long long)img * c_out + co] >= need) bits |= 1u << b;
  }
  mask[i] = bits;
}

hipError_t launch_chan_mask(const uint32_t* counts, int n, int c_out, int words, uint32_t need, uint32_t* mask,
                            hipStream_t s) {
  const int total = n * words;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(chan_mask_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, counts, n, c_out,
                     words, need, mask);
  return hipGetLastError();
}

hipError_t launch_zero_u32(uint32_t* ptr, size_t words, hipStream_t s) {
  if (words == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((words + 255) / 256);
  hipLaunchKernelGGL(zero_u32_kernel, dim3(blocks), dim3(256), 0, s, ptr, words);
  return hipGetLastError();
}

hipError_t launch_naive(const Params& p, hipStream_t s) {
  const long long threads = p.m_total * (long long)p.words * 32;
  if (threads == 0) return hipSuccess;
  const long long blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  dim3 g((unsigned)blocks), b(256);
  switch (p.in_dtype) {
    case CG_F32: hipLaunchKernelGGL(naive_kernel<float>, g, b, 0, s, p); break;
    case CG_BF16: hipLaunchKernelGGL(naive_kernel<uint16_t>, g, b, 0, s, p); break;
    case CG_I8: hipLaunchKernelGGL(naive_kernel<int8_t>, g, b, 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace cg
