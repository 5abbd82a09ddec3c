// Matrix-core kernels of the gated convolution (bf16 -> fp32 and int8 -> int32 MFMA).
//
// One workgroup (4 wavefronts, 2x2) owns a tile of up to 128 output pixels x BN output
// channels and runs the whole layer for it (Eq. 1 of the channel-gating paper):
//
//   phase 0  base path: implicit GEMM over the taps x base channels.  The input patch of
//            the tile and the matching slice of prepacked weights are staged in LDS; every
//            MFMA operand is one 16-byte LDS read (NHWC keeps a tap's channels contiguous).
//   gate     compare the accumulators with the per-channel threshold (merged gate of
//            Sec. 3.2); wavefront ballots give the decision words and tell which 16x16
//            accumulator blocks hold a fired gate.
//   phase 1  conditional path: same GEMM over the remaining channels, accumulated into a
//            second register set; 16-pixel x 16-channel blocks with no fired gate are skipped.
//   output   S = P + d*R goes through LDS so that scale/shift, residual, ReLU, rounding and the
//            stores run on whole pixel rows (coalesced 16-byte accesses).
//
// The dense convolution used as the comparator is the same kernel with c_base == c_in.
#include <cstdlib>

#include "cg_mfma_common.h"

namespace cg {

namespace {

constexpr int kThreads = 256;
constexpr int kBM = 128;       // output pixels per tile, padded
constexpr int kNGW = 4;        // 16-pixel row groups per wavefront
constexpr int kMaxSteps = 20;  // K steps per stage (<= ceil(9*8/4))
constexpr int kMaxTi = 8;      // images per tile

// ---------------------------------------------------------------------------------------
// weight prepack: [c_out][taps][c] -> [column block][stage][e = 4*step + lane group][BN][16 bytes]
// where chunk e of a stage is (tap, q) = (e / cbq, e % cbq); chunks past taps*cbq are zero.
// ---------------------------------------------------------------------------------------
__global__ void pack_weights_kernel(const char* __restrict__ w, char* __restrict__ out, int c_out, int taps, int c_phase,
                                    int eb, int ch, int bn, int cbq, int stages, int tsteps) {
  const long long total = (long long)(c_out / bn) * stages * tsteps * 4 * bn;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int j = (int)(i % bn);
  long long r = i / bn;
  const int e = (int)(r % (tsteps * 4));
  r /= tsteps * 4;
  const int stage = (int)(r % stages);
  const int cbk = (int)(r / stages);
  const int tap = e / cbq, q = e % cbq;
  i32x4 v = {0, 0, 0, 0};
  if (tap < taps) {
    const int co = cbk * bn + j;
    const int c0 = (stage * cbq + q) * ch;
    v = *(const i32x4*)(w + (((long long)co * taps + tap) * c_phase + c0) * eb);
  }
  *(i32x4*)(out + i * 16) = v;
}

// ---------------------------------------------------------------------------------------
// the layer kernel
// ---------------------------------------------------------------------------------------
template <typename Tr, int BN>
__global__ __launch_bounds__(kThreads, 2) void gated_conv_mfma_kernel(Params p, MfmaPlan g, const char* __restrict__ wpk0,
                                                                      const char* __restrict__ wpk1) {
  using acc4 = typename Tr::acc4;
  using acc_t = typename Tr::acc_t;
  constexpr int NBW = BN / 32;       // 16-column fragments per wavefront (2 wavefronts across BN)
  constexpr int LDT = BN + 4;        // row stride (words) of the output tile in LDS

  extern __shared__ __align__(16) char smem[];
  uint32_t* aoff = (uint32_t*)(smem + g.lds_aoff);         // [2][kMaxSteps*4]
  int* pix_gidx = (int*)(smem + g.lds_gidx);               // [npix] input pixel index or -1
  int* out_pp = (int*)(smem + g.lds_outpp);                // [kBM] patch pixel of tap (0,0)
  int* out_m = (int*)(smem + g.lds_outm);                  // [kBM] output pixel index or -1
  uint32_t* colcnt = (uint32_t*)(smem + g.lds_colcnt);     // [ti][BN]
  uint32_t* dbits = (uint32_t*)(smem + g.lds_dbits);       // [kBM][BN/32]
  char* stage_mem = smem + g.lds_stage;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int lj = lane & 15, lg = lane >> 4;

  const int cbk = blockIdx.x % g.n_cb;
  const int tile = blockIdx.x / g.n_cb;
  int img0, row0;
  if (g.ti > 1) {
    img0 = tile * g.ti;
    row0 = 0;
  } else {
    img0 = tile / g.tiles_per_img;
    row0 = (tile - img0 * g.tiles_per_img) * g.tr;
  }

  // ---- per-tile tables -------------------------------------------------------------
  {
    const int ppi = g.pr * g.pwid;
    for (int i = tid; i < g.npix; i += kThreads) {
      const int til = i / ppi, rem = i - til * ppi;
      const int prow = rem / g.pwid, pcol = rem - prow * g.pwid;
      const int img = img0 + til;
      const int hi = row0 * p.stride - p.pad + prow, wi = pcol - p.pad;
      const bool ok = img < p.n && hi >= 0 && hi < p.h && wi >= 0 && wi < p.w;
      pix_gidx[i] = ok ? (img * p.h + hi) * p.w + wi : -1;
    }
    const int opi = g.tr * p.wo;
    for (int i = tid; i < kBM; i += kThreads) {
      int pp = 0, m = -1;
      if (i < g.bm_valid) {
        const int til = i / opi, rem = i - til * opi;
        const int trow = rem / p.wo, wo = rem - trow * p.wo;
        const int img = img0 + til, ho = row0 + trow;
        pp = (til * g.pr + trow * p.stride) * g.pwid + wo * p.stride;
        if (img < p.n && ho < p.ho) m = (img * p.ho + ho) * p.wo + wo;
      }
      out_pp[i] = pp;
      out_m[i] = m;
    }
    for (int i = tid; i < 2 * kMaxSteps * 4; i += kThreads) {
      const int ph = i / (kMaxSteps * 4), e = i - ph * (kMaxSteps * 4);
      uint32_t off = 0;
      if (g.stages[ph] > 0) {
        const int tap = e / g.cbq[ph], q = e - tap * g.cbq[ph];
        if (tap < g.taps) {
          const int r = tap / p.kw, s = tap - r * p.kw;
          off = (uint32_t)((r * g.pwid + s) * g.ps[ph] + q * 16);
        } else {
          off = (uint32_t)(g.cbq[ph] * 16);  // the zero chunk every pixel carries
        }
      }
      aoff[i] = off;
    }
    for (int i = tid; i < g.ti * BN; i += kThreads) colcnt[i] = 0u;
    for (int i = tid; i < kBM * (BN / 32); i += kThreads) dbits[i] = 0u;
  }
  __syncthreads();

  // ---- this wavefront's rows -----------------------------------------------------------
  const int half = (g.ng + 1) >> 1;
  const int base_g = wm * half;
  const int n_groups = wm == 0 ? half : g.ng - half;   // live row groups of this wavefront (<= 4)
  int pix_of[kNGW];
#pragma unroll
  for (int fr = 0; fr < kNGW; ++fr) {
    const int row = (base_g + fr) * 16 + lj;
    pix_of[fr] = out_pp[row < kBM ? row : 0];
  }
  const int col_w = wn * (BN / 2);   // first column of this wavefront inside the tile

  acc4 accP[kNGW][NBW], accR[kNGW][NBW];
#pragma unroll
  for (int fr = 0; fr < kNGW; ++fr)
#pragma unroll
    for (int fc = 0; fc < NBW; ++fc) {
      accP[fr][fc] = acc4{0, 0, 0, 0};
      accR[fr][fc] = acc4{0, 0, 0, 0};
    }

  unsigned act = 0;  // wave-uniform: bit fr*NBW+fc set = block takes part in the current phase
#pragma unroll
  for (int fr = 0; fr < kNGW; ++fr)
    if (fr < n_groups) act |= ((1u << NBW) - 1u) << (fr * NBW);
  unsigned long long dmask = 0;  // per-lane decisions, bit (fr*NBW+fc)*4+i

  const char* xbytes = (const char*)p.x;
  const int eb = g.elem_bytes;

  for (int ph = 0; ph < 2; ++ph) {
    if (g.stages[ph] == 0) continue;
    const int cbq = g.cbq[ph], ps = g.ps[ph], T = g.tsteps[ph];
    const char* wsrc = (ph == 0 ? wpk0 : wpk1) + (size_t)cbk * g.stages[ph] * g.wpk_stage_bytes[ph];
    char* patch = stage_mem;
    char* wl = stage_mem + g.lds_w[ph];
    const uint32_t* ao_tab = aoff + ph * (kMaxSteps * 4);
    int poff[kNGW];
#pragma unroll
    for (int fr = 0; fr < kNGW; ++fr) poff[fr] = pix_of[fr] * ps;

    for (int st = 0; st < g.stages[ph]; ++st) {
      __syncthreads();  // previous stage's reads are done
      {
        // input patch slice: cbq data chunks + one zero chunk per pixel
        const int per = cbq + 1;
        const long long c0 = (long long)(ph ? p.c_base : 0) + (long long)st * cbq * g.ch;
        const int total = g.npix * per;
        for (int i = tid; i < total; i += kThreads) {
          const int pix = i / per, q = i - pix * per;
          i32x4 v = {0, 0, 0, 0};
          const int gi = pix_gidx[pix];
          if (q < cbq && gi >= 0) v = *(const i32x4*)(xbytes + ((long long)gi * p.x_pixel_stride + c0 + q * g.ch) * eb);
          *(i32x4*)(patch + pix * ps + q * 16) = v;
        }
        // weight slice: straight copy of the prepacked image
        const i32x4* src = (const i32x4*)(wsrc + (size_t)st * g.wpk_stage_bytes[ph]);
        const int wchunks = T * 4 * BN;
        for (int i = tid; i < wchunks; i += kThreads) ((i32x4*)wl)[i] = src[i];
      }
      __syncthreads();

      if (act != 0) {
        for (int t = 0; t < T; ++t) {
          const uint32_t ao = ao_tab[t * 4 + lg];
          i32x4 a[kNGW], b[NBW];
#pragma unroll
          for (int fr = 0; fr < kNGW; ++fr) a[fr] = *(const i32x4*)(patch + poff[fr] + ao);
#pragma unroll
          for (int fc = 0; fc < NBW; ++fc)
            b[fc] = *(const i32x4*)(wl + (((t * 4 + lg) * BN) + col_w + fc * 16 + lj) * 16);
#pragma unroll
          for (int fr = 0; fr < kNGW; ++fr)
#pragma unroll
            for (int fc = 0; fc < NBW; ++fc) {
              if (act & (1u << (fr * NBW + fc))) {
                if (ph == 0)
                  accP[fr][fc] = Tr::mfma(a[fr], b[fc], accP[fr][fc]);
                else
                  accR[fr][fc] = Tr::mfma(a[fr], b[fc], accR[fr][fc]);
              }
            }
        }
      }
    }

    // ---- gate (after the base phase of a gated layer) ------------------------------------
    if (ph == 0 && p.gated) {
      acc_t tlo[NBW], thi[NBW];
#pragma unroll
      for (int fc = 0; fc < NBW; ++fc) {
        const int co = cbk * BN + col_w + fc * 16 + lj;
        if constexpr (Tr::kDtype == CG_I8) {
          tlo[fc] = p.thr_i[co];
          thi[fc] = 0;
        } else {
          tlo[fc] = p.thr_f[co];
          thi[fc] = p.thr_hi_f[co];
        }
      }
      unsigned new_act = 0;
#pragma unroll
      for (int fr = 0; fr < kNGW; ++fr) {
        if (fr >= n_groups) continue;
        const int row_base = (base_g + fr) * 16;
        bool rv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) rv[i] = out_m[row_base + 4 * lg + i] >= 0;
        // image index inside the tile of the first and last row of the group (for the counts)
        const int opi = g.tr * p.wo;
        const int til_first = row_base / opi;
        int last_row = row_base + 15;
        if (last_row >= g.bm_valid) last_row = g.bm_valid - 1;
        const int til_last = last_row / opi;
        unsigned long long prev_sel = 0;
#pragma unroll
        for (int fc = 0; fc < NBW; ++fc) {
          unsigned long long mk[4];
          int c = 0;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool f = rv[i] && Tr::fires(accP[fr][fc][i], tlo[fc], thi[fc]);
            mk[i] = __ballot(f);
            if (f) {
              dmask |= 1ull << ((fr * NBW + fc) * 4 + i);
              ++c;
            }
          }
          if ((mk[0] | mk[1] | mk[2] | mk[3]) != 0ull) new_act |= 1u << (fr * NBW + fc);
          // per-(image, channel) counts
          if (til_first == til_last) {
            c += shfl_xor_i(c, 16);
            c += shfl_xor_i(c, 32);
            if (lane < 16 && c) atomicAdd(&colcnt[til_first * BN + col_w + fc * 16 + lj], (uint32_t)c);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if ((dmask >> ((fr * NBW + fc) * 4 + i)) & 1ull) {
                const int til = (row_base + 4 * lg + i) / opi;
                atomicAdd(&colcnt[til * BN + col_w + fc * 16 + lj], 1u);
              }
            }
          }
          // decision words: lane l < 16 assembles the 16 bits of row l from the ballots
          const int li = lane & 3, lgg = (lane >> 2) & 3;
          unsigned long long sel = li == 0 ? mk[0] : li == 1 ? mk[1] : li == 2 ? mk[2] : mk[3];
          sel = (sel >> (16 * lgg)) & 0xffffull;
          if (fc & 1) {
            if (lane < 16)
              dbits[(row_base + lane) * (BN / 32) + ((col_w + fc * 16) >> 5)] = (uint32_t)(prev_sel | (sel << 16));
          } else {
            prev_sel = sel;
          }
        }
      }
      act = (unsigned)__builtin_amdgcn_readfirstlane((int)new_act);
    }
  }

  // ---- output: S through LDS, then whole-row epilogue ------------------------------------
  __syncthreads();
  acc_t* tile_s = (acc_t*)stage_mem;
#pragma unroll
  for (int fr = 0; fr < kNGW; ++fr) {
    if (fr >= n_groups) continue;
#pragma unroll
    for (int fc = 0; fc < NBW; ++fc)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (base_g + fr) * 16 + 4 * lg + i;
        const bool f = (dmask >> ((fr * NBW + fc) * 4 + i)) & 1ull;
        acc_t s = accP[fr][fc][i];
        if (f) s += accR[fr][fc][i];
        tile_s[row * LDT + col_w + fc * 16 + lj] = s;
      }
  }
  __syncthreads();

  const int rows_used = g.ng * 16;
  for (int idx = tid; idx < rows_used * (BN / 8); idx += kThreads) {
    const int row = idx / (BN / 8), c8 = idx - row * (BN / 8);
    const int m = out_m[row];
    if (m < 0) continue;
    const uint32_t dw = dbits[row * (BN / 32) + (c8 >> 2)] >> ((c8 & 3) * 8);
    const int co0 = cbk * BN + c8 * 8;
    const long long o = (long long)m * p.c_out + co0;
    const i32x4 s0 = *(const i32x4*)(tile_s + row * LDT + c8 * 8);
    const i32x4 s1 = *(const i32x4*)(tile_s + row * LDT + c8 * 8 + 4);
    finish_store8<Tr>(p, s0, s1, dw & 0xffu, co0, o);
  }

  if (p.bitmap) {
    for (int idx = tid; idx < rows_used * (BN / 32); idx += kThreads) {
      const int row = idx / (BN / 32), w = idx - row * (BN / 32);
      const int m = out_m[row];
      if (m >= 0) p.bitmap[(long long)m * p.words + cbk * (BN / 32) + w] = dbits[idx];
    }
  }
  if (p.counts && p.gated) {
    unsigned long long mine = 0;
    for (int idx = tid; idx < g.ti * BN; idx += kThreads) {
      const int til = idx / BN, c = idx - til * BN;
      const uint32_t v = colcnt[idx];
      const int img = img0 + til;
      if (v && img < p.n) {
        atomicAdd(&p.counts[2 + (long long)img * p.c_out + cbk * BN + c], v);
        mine += v;
      }
    }
    // wavefront sum, one 64-bit atomic per wavefront that saw anything
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) {
      const unsigned lo = (unsigned)shfl_xor_i((int)(unsigned)(mine & 0xffffffffu), sft);
      mine += lo;
    }
    if (lane == 0 && mine) atomicAdd((unsigned long long*)p.counts, mine);
  }
}

template <typename Tr, int BN>
hipError_t launch_one(const MfmaPlan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  const int n_img_groups = (p.n + g.ti - 1) / g.ti;
  const long long tiles = g.ti > 1 ? n_img_groups : (long long)p.n * g.tiles_per_img;
  const long long blocks = tiles * g.n_cb;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  auto kern = gated_conv_mfma_kernel<Tr, BN>;
  static int attr_set_bytes = 0;
  if (g.lds_total > attr_set_bytes) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, g.lds_total);
    if (e != hipSuccess) return e;
    attr_set_bytes = g.lds_total;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), (size_t)g.lds_total, s, p, g, (const char*)w0,
                     (const char*)w1);
  return hipGetLastError();
}

int div_ceil(int a, int b) { return (a + b - 1) / b; }
int align16(int v) { return (v + 15) & ~15; }

}  // namespace

MfmaPlan mfma_plan(const cg_conv_desc& d) {
  MfmaPlan g{};
  g.ok = 0;
  if (d.in_dtype != CG_BF16 && d.in_dtype != CG_I8) return g;
  if (d.groups > 1 || d.tau_c > 0.0f) return g;   // channel grouping, channel-wise gate: row-tiled and plain kernels only
  if (!((d.kh == 3 && d.kw == 3) || (d.kh == 1 && d.kw == 1))) return g;
  g.elem_bytes = d.in_dtype == CG_BF16 ? 2 : 1;
  g.ch = 16 / g.elem_bytes;
  const int c_cond = d.c_in - d.c_base;
  const long long xps = d.x_pixel_stride ? d.x_pixel_stride : d.c_in;
  if (d.c_base % g.ch || c_cond % g.ch || xps % g.ch) return g;
  if (d.c_out % 64) return g;
  const int ho = (d.h + 2 * d.pad - d.kh) / d.stride + 1, wo = (d.w + 2 * d.pad - d.kw) / d.stride + 1;
  if (wo > kBM) return g;
  if ((long long)d.n_max * d.h * d.w >= (1ll << 31) / 2 || (long long)d.n_max * ho * wo >= (1ll << 31) / 2) return g;
  // residual / output vector accesses need 8-channel groups: c_out % 64 covers it

  g.bn = 64;
  g.n_cb = d.c_out / g.bn;
  g.taps = d.kh * d.kw;

  // tile: whole images when one fits in 128 pixels, otherwise a band of output rows
  if (ho * wo <= kBM) {
    g.ti = kBM / (ho * wo);
    if (g.ti > kMaxTi) g.ti = kMaxTi;
    if (g.ti > d.n_max) g.ti = d.n_max;
    g.tr = ho;
    g.tiles_per_img = 1;
  } else {
    g.ti = 1;
    const int tr_max = kBM / wo;
    g.tiles_per_img = div_ceil(ho, tr_max);
    g.tr = div_ceil(ho, g.tiles_per_img);
  }
  g.pr = (g.tr - 1) * d.stride + d.kh;
  g.pwid = (wo - 1) * d.stride + d.kw;
  g.npix = g.ti * g.pr * g.pwid;
  g.bm_valid = g.ti * g.tr * wo;
  g.ng = div_ceil(g.bm_valid, 16);

  // table area
  int off = 0;
  g.lds_aoff = off;
  off += 2 * kMaxSteps * 4 * 4;
  g.lds_gidx = off;
  off += align16(g.npix * 4);
  g.lds_outpp = off;
  off += kBM * 4;
  g.lds_outm = off;
  off += kBM * 4;
  g.lds_colcnt = off;
  off += align16(g.ti * g.bn * 4);
  g.lds_dbits = off;
  off += kBM * (g.bn / 32) * 4;
  g.lds_stage = off;

  const int budget = 80 * 1024 - off;  // two workgroups per CU
  const int cq[2] = {d.c_base / g.ch, c_cond / g.ch};
  int stage_bytes = 0;
  for (int ph = 0; ph < 2; ++ph) {
    g.stages[ph] = 0;
    g.cbq[ph] = 1;
    g.tsteps[ph] = 0;
    g.ps[ph] = 16;
    g.lds_w[ph] = 0;
    g.wpk_stage_bytes[ph] = 0;
    if (cq[ph] == 0) continue;
    int best = 0;
    for (int c = 1; c <= 8 && c <= cq[ph]; ++c) {
      if (cq[ph] % c) continue;
      const int ts = div_ceil(g.taps * c, 4);
      if (ts > kMaxSteps) continue;
      const int ps = (c + ((c & 1) ? 2 : 1)) * 16;
      const int bytes = align16(g.npix * ps) + ts * 4 * g.bn * 16;
      if (bytes <= budget || c == 1) best = c;
    }
    const int c = best;
    g.cbq[ph] = c;
    g.stages[ph] = cq[ph] / c;
    g.tsteps[ph] = div_ceil(g.taps * c, 4);
    g.ps[ph] = (c + ((c & 1) ? 2 : 1)) * 16;
    g.lds_w[ph] = align16(g.npix * g.ps[ph]);
    g.wpk_stage_bytes[ph] = (size_t)g.tsteps[ph] * 4 * g.bn * 16;
    const int bytes = g.lds_w[ph] + (int)g.wpk_stage_bytes[ph];
    if (bytes > stage_bytes) stage_bytes = bytes;
  }
  const int tile_bytes = kBM * (g.bn + 4) * 4;
  if (tile_bytes > stage_bytes) stage_bytes = tile_bytes;
  g.lds_total = g.lds_stage + stage_bytes;
  if (g.lds_total > 160 * 1024) return g;
  g.wpk_base_bytes = (size_t)g.n_cb * g.stages[0] * g.wpk_stage_bytes[0];
  g.wpk_cond_bytes = (size_t)g.n_cb * g.stages[1] * g.wpk_stage_bytes[1];
  g.ok = 1;
  return g;
}

hipError_t launch_pack_weights(const void* w, void* out, int c_out, int taps, int c_phase, int eb, int ch, int bn,
                               int cbq, int stages, int tsteps, hipStream_t s) {
  const long long total = (long long)(c_out / bn) * stages * tsteps * 4 * bn;
  if (total <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(pack_weights_kernel, dim3(blocks), dim3(256), 0, s, (const char*)w, (char*)out, c_out, taps,
                     c_phase, eb, ch, bn, cbq, stages, tsteps);
  return hipGetLastError();
}

hipError_t launch_mfma_pack(const MfmaPlan& g, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s) {
  for (int ph = 0; ph < 2; ++ph) {
    if (g.stages[ph] == 0) continue;
    hipError_t e = launch_pack_weights(ph == 0 ? p.w_base : p.w_cond, ph == 0 ? wpk_base : wpk_cond, p.c_out, g.taps,
                                       ph == 0 ? p.c_base : p.c_cond, g.elem_bytes, g.ch, g.bn, g.cbq[ph],
                                       g.stages[ph], g.tsteps[ph], s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_mfma(const MfmaPlan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (p.in_dtype == CG_BF16) {
    if (g.bn == 64) return launch_one<Bf16Traits, 64>(g, p, w0, w1, s);
    return launch_one<Bf16Traits, 128>(g, p, w0, w1, s);
  }
  if (g.bn == 64) return launch_one<I8Traits, 64>(g, p, w0, w1, s);
  return launch_one<I8Traits, 128>(g, p, w0, w1, s);
}

}  // namespace cg
