// The dense pieces of a ResNet around the gated layers (the paper evaluates ResNet-18, Sec. 5):
// the input convolution on few channels (7x7 stride 2 on RGB), 3x3 stride-2 max pooling and global
// average pooling followed by the fully connected layer.  None of them is gated.  bf16 activations
// and weights, fp32 accumulation.  (The 1x1 stride-2 shortcut convolutions run through
// cg_conv_create / cg_conv_forward as dense layers, c_base == c_in.)
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "cg_device.h"

namespace cg {
int set_error(int code, const char* fmt, ...);   // defined with the host API
}

namespace {

using cg::bf16_to_float;
using cg::float_to_bf16;

constexpr int kTile = 8;      // output pixels per block edge
constexpr int kCb = 64;       // output channels per block
constexpr int kMaxTaps = 7 * 7 * 4;

// Direct convolution for c_in <= 4.  Block = 8x8 output pixels x 64 output channels, 256 threads:
// thread (px, g) accumulates channels [16g, 16g+16) of pixel px.  A wavefront holds one g and 64
// pixels, so its weight reads are LDS broadcasts and its input reads are one word per lane.
__global__ __launch_bounds__(256) void small_cin_conv_kernel(const uint16_t* __restrict__ x,
                                                             const uint16_t* __restrict__ w,
                                                             const float* __restrict__ scale,
                                                             const float* __restrict__ shift, uint16_t* __restrict__ y,
                                                             int n, int h, int wd, int c_in, int c_out, int k, int stride,
                                                             int pad, int ho, int wo, int relu) {
  extern __shared__ float lds[];
  const int taps = k * k * c_in;
  float* wl = lds;                          // [taps][64]
  const int pe = (kTile - 1) * stride + k;  // patch edge
  float* xl = lds + taps * kCb;             // [pe][pe][c_in]
  const int tid = threadIdx.x;
  const int tiles_w = (wo + kTile - 1) / kTile, tiles_h = (ho + kTile - 1) / kTile;
  int b = blockIdx.x;
  const int tw = b % tiles_w;
  b /= tiles_w;
  const int th = b % tiles_h;
  const int img = b / tiles_h;
  const int cb = blockIdx.y;

  // weights of this channel block: caller layout [c_out][k][k][c_in] -> [tap][channel]
  for (int i = tid; i < taps * kCb; i += 256) {
    const int co = i / taps, t = i - co * taps;
    wl[t * kCb + co] = bf16_to_float(w[(long long)(cb * kCb + co) * taps + t]);
  }
  // input patch, zero outside the image
  const int h0 = th * kTile * stride - pad, w0 = tw * kTile * stride - pad;
  for (int i = tid; i < pe * pe * c_in; i += 256) {
    const int c = i % c_in, q = i / c_in;
    const int pw = q % pe, ph = q / pe;
    const int hi = h0 + ph, wi = w0 + pw;
    float v = 0.0f;
    if (hi >= 0 && hi < h && wi >= 0 && wi < wd) v = bf16_to_float(x[(((long long)img * h + hi) * wd + wi) * c_in + c]);
    xl[i] = v;
  }
  __syncthreads();

  const int px = tid & 63, g = tid >> 6;
  const int oh = px / kTile, ow = px % kTile;
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
  const float* xp = xl + ((oh * stride) * pe + ow * stride) * c_in;
  const int row_taps = k * c_in;            // contiguous taps of one kernel row
  for (int r = 0; r < k; ++r) {
    const float* xr = xp + r * pe * c_in;
    const float* wr = wl + (r * row_taps) * kCb + g * 16;
    for (int t = 0; t < row_taps; ++t) {
      const float xv = xr[t];
      const float4 w0v = *(const float4*)(wr + t * kCb);
      const float4 w1v = *(const float4*)(wr + t * kCb + 4);
      const float4 w2v = *(const float4*)(wr + t * kCb + 8);
      const float4 w3v = *(const float4*)(wr + t * kCb + 12);
      acc[0] = fmaf(xv, w0v.x, acc[0]);
      acc[1] = fmaf(xv, w0v.y, acc[1]);
      acc[2] = fmaf(xv, w0v.z, acc[2]);
      acc[3] = fmaf(xv, w0v.w, acc[3]);
      acc[4] = fmaf(xv, w1v.x, acc[4]);
      acc[5] = fmaf(xv, w1v.y, acc[5]);
      acc[6] = fmaf(xv, w1v.z, acc[6]);
      acc[7] = fmaf(xv, w1v.w, acc[7]);
      acc[8] = fmaf(xv, w2v.x, acc[8]);
      acc[9] = fmaf(xv, w2v.y, acc[9]);
      acc[10] = fmaf(xv, w2v.z, acc[10]);
      acc[11] = fmaf(xv, w2v.w, acc[11]);
      acc[12] = fmaf(xv, w3v.x, acc[12]);
      acc[13] = fmaf(xv, w3v.y, acc[13]);
      acc[14] = fmaf(xv, w3v.z, acc[14]);
      acc[15] = fmaf(xv, w3v.w, acc[15]);
    }
  }
  const int oy = th * kTile + oh, ox = tw * kTile + ow;
  if (oy < ho && ox < wo) {
    const int co0 = cb * kCb + g * 16;
    uint16_t out[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float a = acc[i];
      if (scale) a *= scale[co0 + i];
      if (shift) a += shift[co0 + i];
      if (relu) a = fmaxf(a, 0.0f);
      out[i] = float_to_bf16(a);
    }
    uint4* dst = (uint4*)(y + (((long long)img * ho + oy) * wo + ox) * c_out + co0);
    dst[0] = *(const uint4*)(out);
    dst[1] = *(const uint4*)(out + 8);
  }
}

// The ImageNet input layer's shape (7x7, stride 2, three input channels) on the matrix cores.
// Block = 16x16 output pixels x 64 channels, four wavefronts, each 64 pixels x 64 channels as 2x2
// 32x32 MFMA blocks.  K is ordered kernel row by kernel row; within a row the 21 values (column,
// channel) of a pixel are 21 contiguous bf16 of the input patch, padded to 24 = three 8-element
// chunks (the three extra elements meet zero weights), so the pixel operand of a chunk is 16
// contiguous bytes of the LDS patch, read as four words (the start is only 4-byte aligned).
// 7 rows x 3 chunks = 21 chunks, padded to 22 = 11 K steps of 16.  The product is taken with the
// weights as the row operand and their rows permuted (row rho holds channel
// 16*((rho/4)%2) + 4*(rho/8) + rho%4), which leaves every lane with 16 consecutive channels of
// one pixel per accumulator.
typedef __attribute__((ext_vector_type(8))) __bf16 stem_bf16x8;
typedef __attribute__((ext_vector_type(16))) float stem_f32x16;
typedef __attribute__((ext_vector_type(4))) int stem_i32x4;

//
// POOL: the 3x3 stride-2 max pooling (padding 1) that follows the layer in a ResNet is applied in
// the block: the 16x16 tile then starts one row and column before an even position and yields the
// 7x7 pooled pixels whose windows it holds (neighbouring tiles overlap by two rows / columns); the
// converted outputs meet in an LDS tile, positions outside the layer's output count as -inf, and
// only the pooled tensor is written.
template <bool POOL>
__global__ __launch_bounds__(256) void conv7x7s2c3_mfma_kernel(const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ w,
                                                               const float* __restrict__ scale,
                                                               const float* __restrict__ shift, uint16_t* __restrict__ y,
                                                               int n, int h, int wd, int c_out, int pad, int ho, int wo,
                                                               int relu, int tpb) {
  constexpr int K = 7, CI = 3, ST = 2, TILE = 16, TAPS = K * K * CI;
  constexpr int PE = (TILE - 1) * ST + K;          // 37 patch rows / columns in use
  constexpr int PR = 120;                          // bf16 per patch row (111 in use, the rest zero)
  constexpr int PROWS = PE + 1;                    // one more zero row for the padding chunk
  constexpr int NQ = 22;                           // 8-element K chunks
  __shared__ __align__(16) uint16_t wl[NQ * kCb * 8];    // [chunk][row][8]
  __shared__ __align__(16) uint16_t xl[PROWS * PR];
  __shared__ __align__(16) uint16_t ol[POOL ? TILE * TILE * kCb : 8];   // [tile pixel][64 channels] (POOL)
  constexpr int PT = 7;                            // pooled rows / columns per tile (POOL)
  const int pho = (ho - 1) / 2 + 1, pwo = (wo - 1) / 2 + 1;   // pooled output size (POOL)
  const int tid = threadIdx.x;
  // one block walks tpb tiles of a row: the weights are laid out once per block
  const int tiles_w = POOL ? (pwo + PT - 1) / PT : (wo + TILE - 1) / TILE;
  const int tiles_h = POOL ? (pho + PT - 1) / PT : (ho + TILE - 1) / TILE;
  const int strips = (tiles_w + tpb - 1) / tpb;
  int b = blockIdx.x;
  const int tw0 = (b % strips) * tpb;
  b /= strips;
  const int th = b % tiles_h;
  const int img = b / tiles_h;
  const int cb = blockIdx.y;
  const int tw1 = tw0 + tpb < tiles_w ? tw0 + tpb : tiles_w;

  // weights: chunk q = (kernel row q/3, elements 8*(q%3) .. +8 of its 24), row = permuted channel.
  // A thread lays out one (channel, kernel row): 21 contiguous weights become three chunks, the
  // last three elements zero; the 22nd chunk of every row is zero.
  if (tid < kCb) *(uint4*)(wl + (((NQ - 1) * kCb + tid) << 3)) = uint4{0u, 0u, 0u, 0u};
  {
    const uint16_t* wsrc = w + (long long)cb * kCb * TAPS;
    for (int pr = tid; pr < kCb * K; pr += 256) {
      const int col = pr / K, r = pr - col * K;
      const uint16_t* src = wsrc + col * TAPS + r * (K * CI);
      uint16_t v[24];
#pragma unroll
      for (int e = 0; e < K * CI; ++e) v[e] = src[e];
      v[21] = v[22] = v[23] = 0;
      const int ch = col & 31;
      const int row = (col & 32) + 8 * ((ch & 15) >> 2) + 4 * (ch >> 4) + (ch & 3);   // inverse of the row permutation
      uint16_t* dst = wl + (((3 * r) * kCb + row) << 3);
      *(uint4*)(dst) = *(const uint4*)(v);
      *(uint4*)(dst + kCb * 8) = *(const uint4*)(v + 8);
      *(uint4*)(dst + 2 * kCb * 8) = *(const uint4*)(v + 16);
    }
  }
  const int lane = tid & 63, wave = tid >> 6;
  const int lj = lane & 31, lh = lane >> 5;
  // this lane's pixels: fragment 2*wave + fp covers tile rows 2*(2*wave+fp) and the next
  int pbase[2];
#pragma unroll
  for (int fp = 0; fp < 2; ++fp) {
    const int oh = 2 * (2 * wave + fp) + (lj >> 4), ow = lj & 15;
    pbase[fp] = (oh * ST) * PR + ow * ST * CI;     // element offset of the pixel's window, kernel row 0
  }
  for (int tw = tw0; tw < tw1; ++tw) {
  if (tw > tw0) __syncthreads();                   // the previous tile's patch has been read
  // input patch as bf16, zero outside the image and in the padding
  const int oy0 = POOL ? 2 * PT * th - 1 : th * TILE, ox0 = POOL ? 2 * PT * tw - 1 : tw * TILE;   // the tile's first output pixel
  const int h0 = oy0 * ST - pad, w0 = ox0 * ST - pad;
  // a thread fills one patch pixel (three channels) at a time; 40 pixel positions per row, the ones
  // past the patch edge or outside the image are zero
  constexpr int PPR = PR / CI;
#pragma unroll
  for (int u = 0; u < (PROWS * PPR + 255) / 256; ++u) {
    const int pp = tid + 256 * u;
    const int ph = pp / PPR, pw = pp - ph * PPR;
    const int hi = h0 + ph, wi = w0 + pw;
    uint16_t v0 = 0, v1 = 0, v2 = 0;
    if (pp < PROWS * PPR && ph < PE && pw < PE && hi >= 0 && hi < h && wi >= 0 && wi < wd) {
      const uint16_t* src = x + (((long long)img * h + hi) * wd + wi) * CI;
      v0 = src[0];
      v1 = src[1];
      v2 = src[2];
    }
    if (pp < PROWS * PPR) {
      uint16_t* dst = xl + ph * PR + pw * CI;
      dst[0] = v0;
      dst[1] = v1;
      dst[2] = v2;
    }
  }
  __syncthreads();

  stem_f32x16 acc[2][2];
#pragma unroll
  for (int fp = 0; fp < 2; ++fp)
#pragma unroll
    for (int fc = 0; fc < 2; ++fc)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fp][fc][i] = 0.0f;
#pragma unroll
  for (int st = 0; st < NQ / 2; ++st) {
    const int q = 2 * st + lh;                     // this lane half's chunk of the K step
    const int r = q / 3, j0 = (q % 3) * 8;
    stem_i32x4 a[2], bq[2];
#pragma unroll
    for (int fc = 0; fc < 2; ++fc) a[fc] = *(const stem_i32x4*)(wl + ((q * kCb + 32 * fc + lj) << 3));
#pragma unroll
    for (int fp = 0; fp < 2; ++fp) {
      const uint32_t* src = (const uint32_t*)(xl + pbase[fp] + r * PR + j0);
      bq[fp] = stem_i32x4{(int)src[0], (int)src[1], (int)src[2], (int)src[3]};
    }
#pragma unroll
    for (int fp = 0; fp < 2; ++fp)
#pragma unroll
      for (int fc = 0; fc < 2; ++fc)
        acc[fp][fc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(stem_bf16x8, a[fc]),
                                                              __builtin_bit_cast(stem_bf16x8, bq[fp]), acc[fp][fc], 0, 0, 0);
  }
#pragma unroll
  for (int fp = 0; fp < 2; ++fp) {
    const int oy = oy0 + 2 * (2 * wave + fp) + (lj >> 4), ox = ox0 + (lj & 15);
    const bool inside = oy >= 0 && oy < ho && ox >= 0 && ox < wo;
    if (!POOL && !inside) continue;
#pragma unroll
    for (int fc = 0; fc < 2; ++fc) {
      const int co0 = cb * kCb + 32 * fc + 16 * lh;
      float sc[16], sh[16];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 a4 = scale ? *(const float4*)(scale + co0 + 4 * q4) : float4{1.0f, 1.0f, 1.0f, 1.0f};
        const float4 b4 = shift ? *(const float4*)(shift + co0 + 4 * q4) : float4{0.0f, 0.0f, 0.0f, 0.0f};
        sc[4 * q4] = a4.x, sc[4 * q4 + 1] = a4.y, sc[4 * q4 + 2] = a4.z, sc[4 * q4 + 3] = a4.w;
        sh[4 * q4] = b4.x, sh[4 * q4 + 1] = b4.y, sh[4 * q4 + 2] = b4.z, sh[4 * q4 + 3] = b4.w;
      }
      uint16_t out[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float v = acc[fp][fc][i] * sc[i] + sh[i];
        if (relu) v = fmaxf(v, 0.0f);
        out[i] = (POOL && !inside) ? (uint16_t)0xFF80 : float_to_bf16(v);     // 0xFF80 = -inf
      }
      uint4* dst = POOL ? (uint4*)(ol + ((2 * (2 * wave + fp) + (lj >> 4)) * TILE + (lj & 15)) * kCb + 32 * fc + 16 * lh)
                        : (uint4*)(y + (((long long)img * ho + oy) * wo + ox) * c_out + co0);
      dst[0] = *(const uint4*)(out);
      dst[1] = *(const uint4*)(out + 8);
    }
  }
  if constexpr (POOL) {
    __syncthreads();
    // pooled pixel (py, px) of the tile takes tile rows 2py .. 2py+2 and columns 2px .. 2px+2; a thread
    // takes eight channels of one pooled pixel at a time
    for (int it = tid; it < PT * PT * (kCb / 8); it += 256) {
      const int c8 = it & 7, pp = it >> 3;
      const int py = pp / PT, px = pp - py * PT;
      const int gy = PT * th + py, gx = PT * tw + px;
      if (gy >= pho || gx >= pwo) continue;
      float m[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) m[i] = -__builtin_inff();
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int c = 0; c < 3; ++c) {
          uint16_t v[8];
          *(uint4*)v = *(const uint4*)(ol + ((2 * py + r) * TILE + 2 * px + c) * kCb + c8 * 8);
#pragma unroll
          for (int i = 0; i < 8; ++i) m[i] = fmaxf(m[i], bf16_to_float(v[i]));
        }
      uint16_t o8[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) o8[i] = float_to_bf16(m[i]);
      *(uint4*)(y + (((long long)img * pho + gy) * pwo + gx) * c_out + cb * kCb + c8 * 8) = *(const uint4*)o8;
    }
  }
  }   // tiles of the row
}

// 1x1 convolution with stride (the ResNet shortcut) on the matrix cores: a GEMM of the strided
// pixels (column operand, 16 bytes per lane and K step straight from global memory: a pixel's
// channels are contiguous) with the weights of a 64-channel block (row operand, laid out once
// per block in LDS, rows permuted as in the kernel above).  Block = 128 output pixels x 64
// channels, four wavefronts of 32 pixels each.
__global__ __launch_bounds__(256) void pointwise_conv_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                                             const float* __restrict__ scale,
                                                             const float* __restrict__ shift, uint16_t* __restrict__ y,
                                                             long long m_total, int h, int wd, int c_in, int c_out,
                                                             int stride, int ho, int wo, int relu) {
  extern __shared__ __align__(16) uint16_t wlp[];          // [c_in/8 chunks][64 rows][8]
  const int tid = threadIdx.x;
  const int cb = blockIdx.y;
  const int nq = c_in >> 3;
  for (int i = tid; i < nq * kCb; i += 256) {
    const int col = i / nq, q = i - col * nq;            // consecutive threads read consecutive 16-byte pieces
    const int ch = col & 31;
    const int row = (col & 32) + 8 * ((ch & 15) >> 2) + 4 * (ch >> 4) + (ch & 3);
    *(uint4*)(wlp + ((q * kCb + row) << 3)) = *(const uint4*)(w + ((long long)(cb * kCb + col) * c_in + q * 8));
  }
  __syncthreads();
  const int lane = tid & 63, wave = tid >> 6;
  const int lj = lane & 31, lh = lane >> 5;
  const long long m = (long long)blockIdx.x * 128 + wave * 32 + lj;
  const bool valid = m < m_total;
  const long long mm = valid ? m : 0;
  const int ox = (int)(mm % wo);
  const long long t2 = mm / wo;
  const int oy = (int)(t2 % ho);
  const long long img = t2 / ho;
  const uint16_t* src = x + ((img * h + (long long)oy * stride) * wd + (long long)ox * stride) * c_in + lh * 8;
  stem_f32x16 acc[2];
#pragma unroll
  for (int fc = 0; fc < 2; ++fc)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[fc][i] = 0.0f;
  const int steps = c_in >> 4;
#pragma unroll 4
  for (int st = 0; st < steps; ++st) {
    stem_i32x4 b = {0, 0, 0, 0};
    if (valid) b = *(const stem_i32x4*)(src + st * 16);
    const int q = 2 * st + lh;
#pragma unroll
    for (int fc = 0; fc < 2; ++fc) {
      const stem_i32x4 a = *(const stem_i32x4*)(wlp + ((q * kCb + 32 * fc + lj) << 3));
      acc[fc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(stem_bf16x8, a), __builtin_bit_cast(stem_bf16x8, b),
                                                        acc[fc], 0, 0, 0);
    }
  }
  if (!valid) return;
#pragma unroll
  for (int fc = 0; fc < 2; ++fc) {
    const int co0 = cb * kCb + 32 * fc + 16 * lh;
    uint16_t out[16];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float4 a4 = scale ? *(const float4*)(scale + co0 + 4 * q4) : float4{1.0f, 1.0f, 1.0f, 1.0f};
      const float4 b4 = shift ? *(const float4*)(shift + co0 + 4 * q4) : float4{0.0f, 0.0f, 0.0f, 0.0f};
      const float sc[4] = {a4.x, a4.y, a4.z, a4.w}, sh[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = acc[fc][4 * q4 + e] * sc[e] + sh[e];
        if (relu) v = fmaxf(v, 0.0f);
        out[4 * q4 + e] = float_to_bf16(v);
      }
    }
    uint4* dst = (uint4*)(y + m * c_out + co0);
    dst[0] = *(const uint4*)(out);
    dst[1] = *(const uint4*)(out + 8);
  }
}

// 3x3 stride-2 max pooling with padding 1: the maximum over the taps inside the image.
// One thread per (output pixel, 8 channels).
__global__ __launch_bounds__(256) void maxpool3x3s2_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ y, int n,
                                                           int h, int wd, int c, int ho, int wo) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int c8 = c >> 3;
  const long long total = (long long)n * ho * wo * c8;
  if (t >= total) return;
  const int cc = (int)(t % c8);
  long long q = t / c8;
  const int ox = (int)(q % wo);
  q /= wo;
  const int oy = (int)(q % ho);
  const int img = (int)(q / ho);
  float m[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) m[i] = -__builtin_inff();
  for (int r = 0; r < 3; ++r) {
    const int hi = oy * 2 - 1 + r;
    if (hi < 0 || hi >= h) continue;
    for (int s = 0; s < 3; ++s) {
      const int wi = ox * 2 - 1 + s;
      if (wi < 0 || wi >= wd) continue;
      uint16_t v[8];
      *(uint4*)v = *(const uint4*)(x + (((long long)img * h + hi) * wd + wi) * c + cc * 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) m[i] = fmaxf(m[i], bf16_to_float(v[i]));
    }
  }
  uint16_t out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = float_to_bf16(m[i]);
  *(uint4*)(y + (((long long)img * ho + oy) * wo + ox) * c + cc * 8) = *(const uint4*)out;
}

// Global average pooling over hw positions, then logits = W * mean + bias.  One block of sixteen
// wavefronts per image and 256 classes: the map is averaged by all threads (positions split over
// thread groups, partial sums met in LDS), then every wavefront takes a share of the classes.
__global__ __launch_bounds__(1024) void avgpool_fc_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wfc,
                                                         const float* __restrict__ bias, float* __restrict__ logits,
                                                         int hw, int c, int classes) {
  extern __shared__ float mean[];
  const int img = blockIdx.x;
  const int k0 = blockIdx.y * 256, k1 = k0 + 256 < classes ? k0 + 256 : classes;
  const float inv = 1.0f / (float)hw;
  {
    // thread group g of (blockDim / cpad) takes positions g, g + groups, ...; cpad = channels rounded
    // up to 64; the groups' partial sums sit behind the means in LDS and are added in a fixed order
    float* part = mean + c;                        // [groups][cpad], at most blockDim floats
    const int cpad = (c + 63) & ~63;
    const int groups = (int)blockDim.x / cpad > 0 ? (int)blockDim.x / cpad : 1;
    for (int ch0 = 0; ch0 < c; ch0 += groups > 1 ? c : (int)blockDim.x) {
      // a single group strides over the channels by thread index (threads past cpad would otherwise
      // alias the channels of the first ones); several groups split the positions
      const int ch = groups == 1 ? ch0 + (int)threadIdx.x : (int)threadIdx.x % cpad;
      const int g = groups == 1 ? 0 : (int)threadIdx.x / cpad;
      float s = 0.0f;
      if (ch < c && g < groups)
        for (int p = g; p < hw; p += groups) s += bf16_to_float(x[((long long)img * hw + p) * c + ch]);
      if (groups == 1) {
        if (ch < c) mean[ch] = s * inv;
      } else {
        if (g < groups) part[g * cpad + (int)threadIdx.x % cpad] = s;
        __syncthreads();
        if ((int)threadIdx.x < c) {
          float t = 0.0f;
          for (int gg = 0; gg < groups; ++gg) t += part[gg * cpad + threadIdx.x];
          mean[threadIdx.x] = t * inv;
        }
      }
    }
  }
  __syncthreads();
  // one wavefront per class: lanes stride over the channels, then a butterfly sum
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const bool vec = (c & 7) == 0 && (((uintptr_t)wfc) & 15) == 0;     // a lane takes eight consecutive channels per load
  for (int k = k0 + wave; k < k1; k += nw) {
    float s = 0.0f;
    if (vec) {
      for (int ch = lane * 8; ch < c; ch += 512) {
        uint16_t wv[8];
        *(uint4*)wv = *(const uint4*)(wfc + (long long)k * c + ch);
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(bf16_to_float(wv[e]), mean[ch + e], s);
      }
    } else {
      for (int ch = lane; ch < c; ch += 64) s = fmaf(bf16_to_float(wfc[(long long)k * c + ch]), mean[ch], s);
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) s += __shfl_xor(s, sft, 64);
    if (lane == 0) logits[(long long)img * classes + k] = s + (bias ? bias[k] : 0.0f);
  }
}

}  // namespace

extern "C" {

int cg_small_cin_conv(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                      int32_t h, int32_t wd, int32_t c_in, int32_t c_out, int32_t k, int32_t stride, int32_t pad,
                      int32_t relu, void* hip_stream) {
  if (!x || !w || !y) return cg::set_error(CG_EINVAL, "cg_small_cin_conv: x, w and y must not be NULL");
  if (n < 0 || h <= 0 || wd <= 0) return cg::set_error(CG_EINVAL, "cg_small_cin_conv: bad image size");
  if (c_in < 1 || c_in > 4) return cg::set_error(CG_EUNSUPPORTED, "cg_small_cin_conv: c_in must lie in [1, 4]");
  if (c_out <= 0 || c_out % kCb) return cg::set_error(CG_EUNSUPPORTED, "cg_small_cin_conv: c_out must be a multiple of 64");
  if (k < 1 || k > 7 || !(k & 1)) return cg::set_error(CG_EUNSUPPORTED, "cg_small_cin_conv: kernel size must be odd, at most 7");
  if (stride < 1 || stride > 2 || pad < 0 || pad >= k) return cg::set_error(CG_EINVAL, "cg_small_cin_conv: bad stride or pad");
  if (h + 2 * pad < k || wd + 2 * pad < k) return cg::set_error(CG_EINVAL, "cg_small_cin_conv: kernel larger than the padded input");
  if ((((uintptr_t)y) | ((uintptr_t)scale) | ((uintptr_t)shift)) & 15)
    return cg::set_error(CG_EINVAL, "cg_small_cin_conv: y, scale and shift must be 16-byte aligned");
  if (n == 0) return CG_OK;
  const int ho = (h + 2 * pad - k) / stride + 1, wo = (wd + 2 * pad - k) / stride + 1;
  if (k == 7 && stride == 2 && c_in == 3) {      // the ImageNet input layer: the matrix-core kernel
    // 16x16 tiles per block, along a row: a whole row of tiles (the weight layout is then done once
    // per row) when that still leaves two blocks per CU
    const int tiles_w16 = (wo + 15) / 16;
    const long long rows16 = (long long)n * ((ho + 15) / 16) * (c_out / kCb);
    const int tpb = rows16 >= 512 ? tiles_w16 : 1;
    const long long t16 = (long long)n * ((ho + 15) / 16) * ((tiles_w16 + tpb - 1) / tpb);
    if (t16 > 0x7fffffffll) return cg::set_error(CG_EUNSUPPORTED, "cg_small_cin_conv: too many tiles");
    hipLaunchKernelGGL(conv7x7s2c3_mfma_kernel<false>, dim3((unsigned)t16, (unsigned)(c_out / kCb)), dim3(256), 0,
                       (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w, scale, shift, (uint16_t*)y, n, h, wd,
                       c_out, pad, ho, wo, relu, tpb);
    const hipError_t e7 = hipGetLastError();
    if (e7 != hipSuccess) return cg::set_error(CG_EHIP, "cg_small_cin_conv: %s", hipGetErrorString(e7));
    return CG_OK;
  }
  const long long tiles = (long long)n * ((ho + kTile - 1) / kTile) * ((wo + kTile - 1) / kTile);
  if (tiles > 0x7fffffffll) return cg::set_error(CG_EUNSUPPORTED, "cg_small_cin_conv: too many tiles");
  const int pe = (kTile - 1) * stride + k;
  const size_t lds = ((size_t)k * k * c_in * kCb + (size_t)pe * pe * c_in) * sizeof(float);
  hipLaunchKernelGGL(small_cin_conv_kernel, dim3((unsigned)tiles, (unsigned)(c_out / kCb)), dim3(256), lds,
                     (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w, scale, shift, (uint16_t*)y, n, h, wd,
                     c_in, c_out, k, stride, pad, ho, wo, relu);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return cg::set_error(CG_EHIP, "cg_small_cin_conv: %s", hipGetErrorString(e));
  return CG_OK;
}

int cg_conv7x7s2_maxpool(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                         int32_t h, int32_t wd, int32_t c_out, int32_t pad, int32_t relu, void* hip_stream) {
  if (!x || !w || !y) return cg::set_error(CG_EINVAL, "cg_conv7x7s2_maxpool: x, w and y must not be NULL");
  if (n < 0 || h <= 0 || wd <= 0) return cg::set_error(CG_EINVAL, "cg_conv7x7s2_maxpool: bad image size");
  if (c_out <= 0 || c_out % kCb) return cg::set_error(CG_EUNSUPPORTED, "cg_conv7x7s2_maxpool: c_out must be a multiple of 64");
  if (pad < 0 || pad >= 7) return cg::set_error(CG_EINVAL, "cg_conv7x7s2_maxpool: bad pad");
  if (h + 2 * pad < 7 || wd + 2 * pad < 7) return cg::set_error(CG_EINVAL, "cg_conv7x7s2_maxpool: kernel larger than the padded input");
  if ((((uintptr_t)y) | ((uintptr_t)scale) | ((uintptr_t)shift)) & 15)
    return cg::set_error(CG_EINVAL, "cg_conv7x7s2_maxpool: y, scale and shift must be 16-byte aligned");
  if (n == 0) return CG_OK;
  const int ho = (h + 2 * pad - 7) / 2 + 1, wo = (wd + 2 * pad - 7) / 2 + 1;
  const int pho = (ho - 1) / 2 + 1, pwo = (wo - 1) / 2 + 1;
  const int tiles_w = (pwo + 6) / 7;
  const long long rows = (long long)n * ((pho + 6) / 7) * (c_out / kCb);
  const int tpb = rows >= 512 ? tiles_w : 1;
  const long long blocks = (long long)n * ((pho + 6) / 7) * ((tiles_w + tpb - 1) / tpb);
  if (blocks > 0x7fffffffll) return cg::set_error(CG_EUNSUPPORTED, "cg_conv7x7s2_maxpool: too many tiles");
  hipLaunchKernelGGL(conv7x7s2c3_mfma_kernel<true>, dim3((unsigned)blocks, (unsigned)(c_out / kCb)), dim3(256), 0,
                     (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w, scale, shift, (uint16_t*)y, n, h, wd,
                     c_out, pad, ho, wo, relu, tpb);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return cg::set_error(CG_EHIP, "cg_conv7x7s2_maxpool: %s", hipGetErrorString(e));
  return CG_OK;
}

int cg_pointwise_conv(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                      int32_t h, int32_t wd, int32_t c_in, int32_t c_out, int32_t stride, int32_t relu,
                      void* hip_stream) {
  if (!x || !w || !y) return cg::set_error(CG_EINVAL, "cg_pointwise_conv: x, w and y must not be NULL");
  if (n < 0 || h <= 0 || wd <= 0) return cg::set_error(CG_EINVAL, "cg_pointwise_conv: bad image size");
  if (stride < 1) return cg::set_error(CG_EINVAL, "cg_pointwise_conv: stride must be >= 1");
  if (c_in <= 0 || c_in % 16 || c_in > 512)
    return cg::set_error(CG_EUNSUPPORTED, "cg_pointwise_conv: c_in must be a multiple of 16, at most 512");
  if (c_out <= 0 || c_out % kCb) return cg::set_error(CG_EUNSUPPORTED, "cg_pointwise_conv: c_out must be a multiple of 64");
  if ((((uintptr_t)x) | ((uintptr_t)w) | ((uintptr_t)y) | ((uintptr_t)scale) | ((uintptr_t)shift)) & 15)
    return cg::set_error(CG_EINVAL, "cg_pointwise_conv: x, w, y, scale and shift must be 16-byte aligned");
  if (n == 0) return CG_OK;
  const int ho = (h - 1) / stride + 1, wo = (wd - 1) / stride + 1;
  const long long m_total = (long long)n * ho * wo;
  const long long blocks = (m_total + 127) / 128;
  if (blocks > 0x7fffffffll) return cg::set_error(CG_EUNSUPPORTED, "cg_pointwise_conv: too large");
  hipLaunchKernelGGL(pointwise_conv_kernel, dim3((unsigned)blocks, (unsigned)(c_out / kCb)), dim3(256),
                     (size_t)c_in * kCb * 2, (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w, scale, shift,
                     (uint16_t*)y, m_total, h, wd, c_in, c_out, stride, ho, wo, relu);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return cg::set_error(CG_EHIP, "cg_pointwise_conv: %s", hipGetErrorString(e));
  return CG_OK;
}

int cg_maxpool3x3s2(const void* x, void* y, int32_t n, int32_t h, int32_t wd, int32_t c, void* hip_stream) {
  if (!x || !y) return cg::set_error(CG_EINVAL, "cg_maxpool3x3s2: x and y must not be NULL");
  if (n < 0 || h <= 0 || wd <= 0 || c <= 0) return cg::set_error(CG_EINVAL, "cg_maxpool3x3s2: bad size");
  if (c % 8) return cg::set_error(CG_EUNSUPPORTED, "cg_maxpool3x3s2: c must be a multiple of 8");
  if ((((uintptr_t)x) | ((uintptr_t)y)) & 15) return cg::set_error(CG_EINVAL, "cg_maxpool3x3s2: x and y must be 16-byte aligned");
  if (n == 0) return CG_OK;
  const int ho = (h + 2 - 3) / 2 + 1, wo = (wd + 2 - 3) / 2 + 1;
  const long long total = (long long)n * ho * wo * (c / 8);
  const long long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffll) return cg::set_error(CG_EUNSUPPORTED, "cg_maxpool3x3s2: too large");
  hipLaunchKernelGGL(maxpool3x3s2_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint16_t*)x, (uint16_t*)y, n, h, wd, c, ho, wo);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return cg::set_error(CG_EHIP, "cg_maxpool3x3s2: %s", hipGetErrorString(e));
  return CG_OK;
}

int cg_avgpool_fc(const void* x, const void* wfc, const float* bias, float* logits, int32_t n, int32_t hw, int32_t c,
                  int32_t classes, void* hip_stream) {
  if (!x || !wfc || !logits) return cg::set_error(CG_EINVAL, "cg_avgpool_fc: x, wfc and logits must not be NULL");
  if (n < 0 || hw <= 0 || c <= 0 || classes <= 0) return cg::set_error(CG_EINVAL, "cg_avgpool_fc: bad size");
  if (c > 11264) return cg::set_error(CG_EUNSUPPORTED, "cg_avgpool_fc: at most 11264 channels");
  if (n == 0) return CG_OK;
  hipLaunchKernelGGL(avgpool_fc_kernel, dim3((unsigned)n, (unsigned)((classes + 255) / 256)), dim3(1024),
                     ((size_t)c + 1024) * sizeof(float), (hipStream_t)hip_stream,
                     (const uint16_t*)x, (const uint16_t*)wfc, bias, logits, hw, c, classes);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return cg::set_error(CG_EHIP, "cg_avgpool_fc: %s", hipGetErrorString(e));
  return CG_OK;
}

}  // extern "C"
