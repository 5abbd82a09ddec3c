// Pixel-compacting matrix-core kernel of the gated convolution (bf16 and int8 MFMA).
//
// One workgroup (4 wavefronts) owns up to BM = 128 or 256 consecutive output pixels (whole
// output rows of the batch, numbered R = img*Ho + ho, possibly straddling images) times 64
// output channels, and runs the whole layer for them (Eq. 1 of the channel-gating paper):
//
//   base path   implicit GEMM over taps x base channels; wavefront w owns pixel groups
//               [w*NGW, (w+1)*NGW) x all 64 channels (a 64x64 or 32x64 accumulator tile).
//   gate        accumulators against the per-channel threshold (merged gate, Sec. 3.2); ballots
//               give the decision words and a per-pixel "some gate fired" flag.
//   compaction  the pixels with a fired gate are listed with a wavefront prefix sum; only those
//               rows are multiplied on the conditional path.  The A operand of every MFMA is
//               gathered from the LDS-resident input patch by per-lane address, so a compacted
//               row costs the same as a dense one.
//   cond. path  GEMM over taps x remaining channels on the compacted rows (compacted group c
//               goes to wavefront c % 4), into a second accumulator set.
//   output      P (tile rows) and R (compacted rows) meet in LDS; S = P + d*R, scale/shift,
//               residual, ReLU and the stores run on whole pixel rows.
//
// K is consumed in stages of CBQ 16-byte channel chunks per pixel.  Stage s+1 is fetched with
// LDS-direct loads (global_load_lds_dwordx4) into the second buffer while stage s is multiplied.
// The patch is stored as CBQ planes [chunk][pixel], 16 bytes per pixel: the 16 lanes of one lane
// group of an operand read (16 consecutive pixels, one chunk) then cover 256 contiguous bytes and
// the four lane groups sit a multiple of 256 bytes apart, the pattern the LDS serves at full
// rate; operand addresses are additive (pixel + chunk plane + tap offset).  Each plane ends
// in a zero pixel that the K padding reads.
#include <cstdlib>

#include "cg_mfma_common.h"

namespace cg {

namespace {

constexpr int kWaves = 8;              // wavefronts per workgroup: two per SIMD, so that one wavefront's
                                       // LDS / global issue overlaps the other's MFMAs
constexpr int kThreads = kWaves * 64;
constexpr int kBN = 64;
constexpr int kKP = 8;    // patch chunk slots per thread per stage, at most
// Static LDS: two stage buffers and one table area, three separate objects so that the compiler's
// alias analysis keeps LDS-direct loads into one buffer from stalling reads of the other.
constexpr int kStageBytes = 72 * 1024;
constexpr int kTabBytes = 16 * 1024;

// exact x / d for x < 65536, d < 65536, with magic = 2^32 / d rounded up
__device__ __forceinline__ int fdiv(int x, unsigned magic) { return (int)__umulhi((unsigned)x, magic); }

__device__ __forceinline__ void lds_direct_16(const char* gsrc, char* ldst) {
  // each active lane copies 16 bytes from its own global address to ldst + lane*16
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)ldst, 16, 0, 0);
}

template <int CBQ>
struct StageGeom {
  static constexpr int T = (9 * CBQ + 3) / 4;                  // MFMA K steps per stage
};

// One K stage of MFMAs for this wavefront: NRL pixel groups x four 16-channel fragments.
// K step t multiplies chunk e = 4t + lg of the stage (tap e / CBQ, channel chunk e % CBQ);
// arow[fr] is the lane's patch offset of group fr (pixel + chunk plane), aoff[t] the tap offset
// (negative for the K padding past the ninth tap, which reads the zero pixel at zaddr).
// A wavefront issues in order, so the LDS reads of step t+1 (and a slice of the next stage's
// global->LDS loads, issue(t)) are interleaved one by one between the MFMAs of step t; the
// scheduling barriers pin that order.
template <typename Tr, int CBQ, int NRL, int NRMAX, typename IssueFn>
__device__ __forceinline__ void mma_stage(const char* __restrict__ patch, const char* __restrict__ wb,
                                          const int (&arow)[NRMAX], const int (&aoff)[StageGeom<CBQ>::T], int zaddr,
                                          typename Tr::acc4 (&acc)[NRMAX][4], IssueFn&& issue) {
  constexpr int T = StageGeom<CBQ>::T;
  auto a_addr = [&](int fr, int t) __attribute__((always_inline)) {
    if constexpr (CBQ == 4) return arow[fr] + aoff[t];
    return aoff[t] >= 0 ? arow[fr] + aoff[t] : zaddr;
  };
  constexpr int R = NRL + 4;      // operand reads per K step
  constexpr int M = NRL * 4;      // MFMAs per K step
  i32x4 a[2][NRL], b[2][4];
#pragma unroll
  for (int fr = 0; fr < NRL; ++fr) a[0][fr] = *(const i32x4*)(patch + a_addr(fr, 0));
#pragma unroll
  for (int fc = 0; fc < 4; ++fc) b[0][fc] = *(const i32x4*)(wb + fc * 256);
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const int cur = t & 1, nxt = cur ^ 1;
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): operands of step t are in registers
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      if (t + 1 < T) {
        if (i < NRL)
          a[nxt][i] = *(const i32x4*)(patch + a_addr(i, t + 1));
        else
          b[nxt][i - NRL] = *(const i32x4*)(wb + (t + 1) * (4 * kBN * 16) + (i - NRL) * 256);
      }
      if (i == 1) issue(t);
#pragma unroll
      for (int j = (i * M) / R; j < ((i + 1) * M) / R; ++j)
        acc[j >> 2][j & 3] = Tr::mfma(a[cur][j >> 2], b[cur][j & 3], acc[j >> 2][j & 3]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// dispatch on the (workgroup-uniform) number of pixel groups per wavefront
template <typename Tr, int CBQ, int NRMAX, typename IssueFn>
__device__ __forceinline__ void mma_dispatch(int nr, const char* patch, const char* wb, const int (&arow)[NRMAX],
                                             const int (&aoff)[StageGeom<CBQ>::T], int zaddr,
                                             typename Tr::acc4 (&acc)[NRMAX][4], IssueFn&& issue) {
  switch (nr) {
    case 1: mma_stage<Tr, CBQ, 1, NRMAX>(patch, wb, arow, aoff, zaddr, acc, issue); break;
    case 2: if constexpr (NRMAX >= 2) mma_stage<Tr, CBQ, 2, NRMAX>(patch, wb, arow, aoff, zaddr, acc, issue); break;
    default:
#pragma unroll
      for (int t = 0; t < StageGeom<CBQ>::T; ++t) issue(t);
      break;
  }
}

template <typename Tr, int NGW, int CBQ>
__global__ __launch_bounds__(kThreads, 1) void gated_conv_compact_kernel(Params p, Mfma2Plan g,
                                                                         const char* __restrict__ wpk0,
                                                                         const char* __restrict__ wpk1) {
  using acc4 = typename Tr::acc4;
  using acc_t = typename Tr::acc_t;
  using SG = StageGeom<CBQ>;
  constexpr int BM = NGW * 16 * kWaves;
  constexpr int WROWS = (StageGeom<CBQ>::T * 256 + kThreads - 1) / kThreads;   // wave-wide rows of a weight stage slab
  constexpr int T = SG::T;
  constexpr int LOGC = CBQ == 4 ? 2 : CBQ == 2 ? 1 : 0;

  __shared__ __align__(16) char bufA[kStageBytes];
  __shared__ __align__(16) char bufB[kStageBytes];
  __shared__ __align__(16) char smem[kTabBytes];
  int* pix_goff = (int*)(smem + g.lds_goff);             // [npix] input pixel index or -1
  int* out_pp = (int*)(smem + g.lds_outpp);              // [BM] patch pixel of tap (0,0)
  int* out_m = (int*)(smem + g.lds_outm);                // [BM] output pixel index or -1
  int* flag = (int*)(smem + g.lds_flag);                 // [BM] some gate of the pixel fired
  int* clist = (int*)(smem + g.lds_clist);               // [BM] compacted position -> tile row
  int* rank = (int*)(smem + g.lds_rank);                 // [BM] tile row -> compacted position
  uint32_t* dbits = (uint32_t*)(smem + g.lds_dbits);     // [BM][2] decisions of the 64 channels
  uint32_t* colcnt = (uint32_t*)(smem + g.lds_colcnt);   // [max_imgs][64]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lj = lane & 15, lg = lane >> 4;

  // blocks that share a pixel tile (different channel blocks) sit on the same XCD (block id mod 8)
  int tile, cbk;
  {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int grp = slot / g.n_cb;
    cbk = slot - grp * g.n_cb;
    tile = grp * 8 + xcd;
  }
  const int total_rows = p.n * p.ho;
  if (tile * g.tr >= total_rows) return;
  const int R0 = tile * g.tr;
  const int img0 = fdiv(R0, g.magic_ho);
  const int base0 = img0 * g.hp + (R0 - img0 * p.ho) * p.stride;   // stacked padded input row of patch row 0

  // ---- per-tile tables: patch rows over wavefronts, patch columns over lanes ---------------------
  for (int prow = wave; prow < g.pr_max; prow += kWaves) {
    const int srow = base0 + prow;
    const int img = fdiv(srow, g.magic_hp);
    const int hi = srow - img * g.hp - p.pad;
    const bool row_ok = img < p.n && hi >= 0 && hi < p.h;
    const int rowbase = (img * p.h + hi) * p.w - p.pad;
    for (int pcol = lane; pcol < g.pw; pcol += 64) {
      const int wi = pcol - p.pad;
      pix_goff[prow * g.pw + pcol] = (row_ok && wi >= 0 && wi < p.w) ? rowbase + pcol : -1;
    }
  }
  for (int i = tid; i < BM; i += kThreads) {
    int pp = 0, m = -1;
    if (i < g.bm_valid) {
      const int rr = fdiv(i, g.magic_wo), wo = i - rr * p.wo;
      const int R = R0 + rr;
      if (R < total_rows) {
        const int img = fdiv(R, g.magic_ho), hq = R - img * p.ho;
        pp = (img * g.hp + hq * p.stride - base0) * g.pw + wo * p.stride;
        m = R * p.wo + wo;
      }
    }
    out_pp[i] = pp;
    out_m[i] = m;
    flag[i] = 0;
    rank[i] = 0;
    clist[i] = 0;
    dbits[2 * i] = 0u;
    dbits[2 * i + 1] = 0u;
  }
  for (int i = tid; i < g.max_imgs * kBN; i += kThreads) colcnt[i] = 0u;
  __syncthreads();

  // ---- this thread's load slots: slot ci = k*threads + tid of the patch is (chunk plane ci / nps,
  // pixel ci % nps); nps slots per plane, the ones past npix stay zero
  const char* xbytes = (const char*)p.x;
  const int eb = g.elem_bytes;
  int gsl[kKP];
  {
    int gi[kKP], qq[kKP];
    const int last_slot = CBQ * g.nps - 1;
#pragma unroll
    for (int k = 0; k < kKP; ++k) {       // all table reads first, so that their latencies overlap
      int ci = k * kThreads + tid;
      ci = ci > last_slot ? last_slot : ci;
      qq[k] = fdiv(ci, g.magic_nps);
      const int pix = ci - qq[k] * g.nps;
      gi[k] = pix < g.npix ? pix_goff[pix] : -1;
    }
#pragma unroll
    for (int k = 0; k < kKP; ++k) {
      gsl[k] = -1;
      const int ci = k * kThreads + tid;
      if (k < g.kp && ci <= last_slot) {
        if (gi[k] >= 0) {
          gsl[k] = (gi[k] * (int)p.x_pixel_stride + qq[k] * g.ch) * eb;   // the plan keeps x below 2 GiB
        } else {
          // outside the image, or plane padding (the zero pixel): zero once, never written again
          *(i32x4*)(bufA + ci * 16) = i32x4{0, 0, 0, 0};
          *(i32x4*)(bufB + ci * 16) = i32x4{0, 0, 0, 0};
        }
      }
    }
  }

  const int S0 = g.stages[0];
  int S = S0 + (p.gated ? g.stages[1] : 0);

  // slice t (of T) of the loads of stage s: weight K-step slab t and the patch slots k = t, t+T, ...
  auto issue_part = [&](int s, char* pdst, int t) __attribute__((always_inline)) {
    const int ph = s >= S0 ? 1 : 0;
    const int ss = ph ? s - S0 : s;
    char* wdst = pdst + g.patch_bytes;
    const char* ws = (ph ? wpk1 : wpk0) + ((size_t)cbk * g.stages[ph] + ss) * g.wpk_stage_bytes;
    if (t < WROWS) {
      if (t * kThreads + tid < T * 256)
        lds_direct_16(ws + (t * kThreads + tid) * 16, wdst + (t * kThreads + wave * 64) * 16);
    }
    const char* xs = xbytes + (long long)((ph ? p.c_base : 0) + ss * CBQ * g.ch) * eb;
#pragma unroll
    for (int k = 0; k < kKP; ++k) {
      if (k % T == t && k < g.kp) {
        if (gsl[k] >= 0) lds_direct_16(xs + gsl[k], pdst + (k * kThreads + wave * 64) * 16);
      }
    }
  };
  auto issue_stage = [&](int s, char* pdst) __attribute__((always_inline)) {
    const int ph = s >= S0 ? 1 : 0;
    const int ss = ph ? s - S0 : s;
    char* wdst = pdst + g.patch_bytes;
    const char* ws = (ph ? wpk1 : wpk0) + ((size_t)cbk * g.stages[ph] + ss) * g.wpk_stage_bytes;
#pragma unroll
    for (int t = 0; t < WROWS; ++t) {
      if (t * kThreads + tid < T * 256)
        lds_direct_16(ws + (t * kThreads + tid) * 16, wdst + (t * kThreads + wave * 64) * 16);
    }
    const char* xs = xbytes + (long long)((ph ? p.c_base : 0) + ss * CBQ * g.ch) * eb;
#pragma unroll
    for (int k = 0; k < kKP; ++k) {
      if (k < g.kp) {
        if (gsl[k] >= 0) lds_direct_16(xs + gsl[k], pdst + (k * kThreads + wave * 64) * 16);
      }
    }
  };

  // ---- per-lane K-step geometry: chunk e = 4t + lg is (tap, q) = (e / CBQ, e % CBQ) -----------------
  // byte offset of the tap inside plane q; the K padding reads the plane's zero pixel
  const int q = lg & (CBQ - 1);
  const int zaddr = q * g.pln + g.npix * 16;
  int aoff[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const int tap = (4 * t + lg) >> LOGC;
    aoff[t] = tap < 9 ? ((tap / 3) * g.pw + (tap % 3)) * 16 : -1;
  }

  // ---- base-path rows of this wavefront --------------------------------------------------------------
  int ngrp = g.ng - wave * NGW;      // live pixel groups of this wavefront
  ngrp = ngrp < 0 ? 0 : (ngrp > NGW ? NGW : ngrp);
  int arow[NGW], arow_c[NGW];
#pragma unroll
  for (int fr = 0; fr < NGW; ++fr) {
    arow[fr] = out_pp[(wave * NGW + fr) * 16 + lj] * 16 + q * g.pln;
    arow_c[fr] = q * g.pln;
  }

  acc4 accP[NGW][4], accR[NGW][4];
#pragma unroll
  for (int fr = 0; fr < NGW; ++fr)
#pragma unroll
    for (int fc = 0; fc < 4; ++fc) {
      accP[fr][fc] = acc4{0, 0, 0, 0};
      accR[fr][fc] = acc4{0, 0, 0, 0};
    }

  int nrc = 0;                    // live compacted groups of this wavefront
  int nr_wg = 0;                  // compacted groups every wavefront multiplies = ceil(groups / 4)
  const int wlane = (lg * kBN + lj) * 16;   // lane's offset inside a weight K-step slab

  // gate thresholds of this lane's four channels, fetched before any prefetch is in flight
  // (a later global load would queue behind the stage loads)
  acc_t tlo[4], thi[4];
#pragma unroll
  for (int fc = 0; fc < 4; ++fc) {
    const int co = cbk * kBN + fc * 16 + lj;
    if constexpr (Tr::kDtype == CG_I8) {
      tlo[fc] = p.gated ? p.thr_i[co] : 0;
      thi[fc] = 0;
    } else {
      tlo[fc] = p.gated ? p.thr_f[co] : 0.0f;
      thi[fc] = p.gated ? p.thr_hi_f[co] : 0.0f;
    }
  }

  issue_stage(0, bufA);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the LDS-direct loads have landed
  __syncthreads();

  // one K stage: prefetch the next stage into `nxt`, multiply out of `cur`
  auto do_stage = [&](int s, const char* cur, char* nxt) __attribute__((always_inline)) {
    const bool prefetch = s + 1 < S;
    auto part = [&](int t) __attribute__((always_inline)) {
      if (prefetch) issue_part(s + 1, nxt, t);
    };
    const char* patch = cur;
    const char* wb = cur + g.patch_bytes + wlane;
    if (s < S0) {
      // every wavefront multiplies NGW groups: the ones past the tile's end read pixel 0 and are dropped
      mma_stage<Tr, CBQ, NGW, NGW>(patch, wb, arow, aoff, zaddr, accP, part);
    } else {
      mma_dispatch<Tr, CBQ, NGW>(nr_wg, patch, wb, arow_c, aoff, zaddr, accR, part);
    }

    if (s == S0 - 1 && p.gated) {
      // ---- gate ------------------------------------------------------------------------------
      // images (relative to img0) of this wavefront's first and last live pixel
      int last_row = (wave * NGW + ngrp) * 16 - 1;
      if (last_row >= g.bm_valid) last_row = g.bm_valid - 1;
      const int il0 = fdiv(R0 + fdiv(wave * NGW * 16, g.magic_wo), g.magic_ho) - img0;
      const int il1 = ngrp > 0 ? fdiv(R0 + fdiv(last_row, g.magic_wo), g.magic_ho) - img0 : il0;
      int cnt[4] = {0, 0, 0, 0};   // fired gates of this lane per channel fragment
      unsigned dm = 0;             // this lane's decisions, bit fr*16 + fc*4 + i
      const int li = lane & 3, lgg = (lane >> 2) & 3;   // lanes 0..15 assemble the decision words of row `lane`
#pragma unroll
      for (int fr = 0; fr < NGW; ++fr) {
        if (fr >= ngrp) continue;
        const int row_base = (wave * NGW + fr) * 16;
        unsigned vm = 0;           // bit i: pixel 4*lg+i is a real output pixel
#pragma unroll
        for (int i = 0; i < 4; ++i) vm |= (out_m[row_base + 4 * lg + i] >= 0 ? 1u : 0u) << i;
        const unsigned long long vball[4] = {__ballot(vm & 1u), __ballot(vm & 2u), __ballot(vm & 4u), __ballot(vm & 8u)};
        unsigned d16 = 0;          // this lane's 16 decisions of the group, bit fc*4 + i
        unsigned prev_sel = 0;
#pragma unroll
        for (int fc = 0; fc < 4; ++fc) {
          unsigned long long mk[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool f = Tr::fires(accP[fr][fc][i], tlo[fc], thi[fc]);
            mk[i] = __ballot(f) & vball[i];
            d16 |= (f ? 1u : 0u) << (fc * 4 + i);
          }
          // bits 16*g .. 16*g+15 of ballot i are the 16 channels of pixel 4*g+i
          const unsigned long long m64 = li == 0 ? mk[0] : li == 1 ? mk[1] : li == 2 ? mk[2] : mk[3];
          const unsigned half = lgg < 2 ? (unsigned)m64 : (unsigned)(m64 >> 32);
          const unsigned sel = (half >> (16 * (lgg & 1))) & 0xffffu;
          if (fc & 1) {
            if (lane < 16) dbits[(row_base + lane) * 2 + (fc >> 1)] = prev_sel | (sel << 16);
          } else {
            prev_sel = sel;
          }
        }
        d16 &= vm * 0x1111u;       // drop the rows past the end of the tile
        dm |= d16 << (fr * 16);
        const unsigned anyb = (d16 | (d16 >> 4) | (d16 >> 8) | (d16 >> 12)) & 0xfu;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned long long b = __ballot((anyb >> i) & 1u);
          const unsigned half = lg < 2 ? (unsigned)b : (unsigned)(b >> 32);
          if (lj == 0) flag[row_base + 4 * lg + i] = ((half >> (16 * (lg & 1))) & 0xffffu) != 0u;
        }
      }
#pragma unroll
      for (int fc = 0; fc < 4; ++fc) {
        unsigned msk = 0;
#pragma unroll
        for (int fr = 0; fr < NGW; ++fr) msk |= 0xfu << (fr * 16 + fc * 4);
        cnt[fc] = __popc(dm & msk);
      }
      // per-(image, channel) counts: one LDS atomic per fragment when the wavefront sits in one image
      if (il0 == il1) {
#pragma unroll
        for (int fc = 0; fc < 4; ++fc)
          if (cnt[fc]) atomicAdd(&colcnt[il0 * kBN + fc * 16 + lj], (uint32_t)cnt[fc]);
      } else {
#pragma nounroll
        for (int e = 0; e < NGW * 16; ++e) {
          if ((dm >> e) & 1u) {
            const int row = (wave * NGW + (e >> 4)) * 16 + 4 * lg + (e & 3);
            const int il = fdiv(R0 + fdiv(row, g.magic_wo), g.magic_ho) - img0;
            atomicAdd(&colcnt[il * kBN + ((e >> 2) & 3) * 16 + lj], 1u);
          }
        }
      }
      __syncthreads();

      // ---- compaction: every wavefront scans all flags, thread r places row r ----------------------
      int n_act = 0, my_prefix = 0;
      unsigned long long my_bal = 0;
#pragma unroll
      for (int c = 0; c < BM / 64; ++c) {
        const unsigned long long b = __ballot(flag[c * 64 + lane] != 0);
        if (c == wave) {
          my_prefix = n_act;
          my_bal = b;
        }
        n_act += __popcll(b);
      }
      if (tid < BM && ((my_bal >> lane) & 1ull)) {
        const int idx = my_prefix + __popcll(my_bal & ((1ull << lane) - 1ull));
        clist[idx] = tid;
        rank[tid] = idx;
      }
      __syncthreads();

      // compacted group c (16 rows) goes to wavefront c % kWaves
      const int ngc = (n_act + 15) >> 4;
      nrc = ngc > wave ? (ngc - wave + kWaves - 1) / kWaves : 0;
      nr_wg = (ngc + kWaves - 1) / kWaves;
#pragma unroll
      for (int fr = 0; fr < NGW; ++fr) {
        const int c = (wave + kWaves * fr) * 16 + lj;
        arow_c[fr] = out_pp[c < n_act ? clist[c] : 0] * 16 + q * g.pln;
      }
      if (n_act == 0) S = s + 1;   // nothing fired in this tile: the conditional stages are skipped
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  };

  for (int s = 0; s < S; s += 2) {
    do_stage(s, bufA, bufB);
    if (s + 1 < S) do_stage(s + 1, bufB, bufA);
  }

  // ---- output: P by tile row, R by compacted row, both through LDS ---------------------------------
  acc_t* tileP = (acc_t*)bufA;
  acc_t* tileR = (acc_t*)bufB;
#pragma unroll
  for (int fr = 0; fr < NGW; ++fr) {
    if (fr >= ngrp) continue;
#pragma unroll
    for (int fc = 0; fc < 4; ++fc)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (wave * NGW + fr) * 16 + 4 * lg + i;
        tileP[row * kBN + ((fc * 16 + lj) ^ (lg << 4))] = accP[fr][fc][i];
      }
  }
  if (p.gated) {
#pragma unroll
    for (int fr = 0; fr < NGW; ++fr) {
      if (fr >= nrc) continue;
#pragma unroll
      for (int fc = 0; fc < 4; ++fc)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int crow = (wave + kWaves * fr) * 16 + 4 * lg + i;
          tileR[crow * kBN + ((fc * 16 + lj) ^ (lg << 4))] = accR[fr][fc][i];
        }
    }
  }
  __syncthreads();

  const int rows_used = g.ng * 16;
#pragma unroll 4
  for (int idx = tid; idx < rows_used * 8; idx += kThreads) {
    const int row = idx >> 3, c8 = idx & 7;
    const int m = out_m[row];
    if (m < 0) continue;
    const uint32_t db = (dbits[row * 2 + (c8 >> 2)] >> ((c8 & 3) * 8)) & 0xffu;
    const int co0 = cbk * kBN + c8 * 8;
    const long long o = (long long)m * p.c_out + co0;
    const acc_t* pp = tileP + row * kBN + ((c8 * 8) ^ (((row >> 2) & 3) << 4));
    i32x4 s0 = *(const i32x4*)pp;
    i32x4 s1 = *(const i32x4*)(pp + 4);
    if (db) {
      const int cr = rank[row];
      const acc_t* rp = tileR + cr * kBN + ((c8 * 8) ^ (((cr >> 2) & 3) << 4));
      const i32x4 r0 = *(const i32x4*)rp;
      const i32x4 r1 = *(const i32x4*)(rp + 4);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const bool on = (db >> k) & 1u;
        if constexpr (Tr::kDtype == CG_I8) {
          const int r = on ? (k < 4 ? r0[k] : r1[k - 4]) : 0;
          if (k < 4) s0[k] += r; else s1[k - 4] += r;
        } else {
          const float r = on ? __int_as_float(k < 4 ? r0[k] : r1[k - 4]) : 0.0f;
          if (k < 4)
            s0[k] = __float_as_int(__int_as_float(s0[k]) + r);
          else
            s1[k - 4] = __float_as_int(__int_as_float(s1[k - 4]) + r);
        }
      }
    }
    finish_store8<Tr>(p, s0, s1, db, co0, o);
  }

  if (p.bitmap) {
    for (int idx = tid; idx < rows_used * 2; idx += kThreads) {
      const int row = idx >> 1, w = idx & 1;
      const int m = out_m[row];
      if (m >= 0) p.bitmap[(long long)m * p.words + cbk * 2 + w] = dbits[idx];
    }
  }
  if (p.counts && p.gated) {
    unsigned long long mine = 0;
    for (int idx = tid; idx < g.max_imgs * kBN; idx += kThreads) {
      const int il = idx >> 6, c = idx & 63;
      const uint32_t v = colcnt[idx];
      const int img = img0 + il;
      if (v && img < p.n) {
        atomicAdd(&p.counts[2 + (long long)img * p.c_out + cbk * kBN + c], v);
        mine += v;
      }
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) mine += (unsigned)shfl_xor_i((int)(unsigned)(mine & 0xffffffffu), sft);
    if (lane == 0 && mine) atomicAdd((unsigned long long*)p.counts, mine);
  }
}

template <typename Tr, int NGW, int CBQ>
hipError_t launch_one(const Mfma2Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  const long long rows = (long long)p.n * p.ho;
  const long long tiles = (rows + g.tr - 1) / g.tr;
  const long long blocks = ((tiles + 7) / 8) * 8 * g.n_cb;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  auto kern = gated_conv_compact_kernel<Tr, NGW, CBQ>;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), 0, s, p, g, (const char*)w0, (const char*)w1);
  return hipGetLastError();
}

template <typename Tr>
hipError_t launch_dtype(const Mfma2Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (g.ngw == 2) {
    if (g.cbq == 4) return launch_one<Tr, 2, 4>(g, p, w0, w1, s);
    if (g.cbq == 2) return launch_one<Tr, 2, 2>(g, p, w0, w1, s);
    return launch_one<Tr, 2, 1>(g, p, w0, w1, s);
  }
  if (g.cbq == 4) return launch_one<Tr, 1, 4>(g, p, w0, w1, s);
  if (g.cbq == 2) return launch_one<Tr, 1, 2>(g, p, w0, w1, s);
  return launch_one<Tr, 1, 1>(g, p, w0, w1, s);
}

int align_up(int v, int a) { return (v + a - 1) / a * a; }
unsigned magic_of(int d) { return (unsigned)(((1ull << 32) + (unsigned)d - 1) / (unsigned)d); }

}  // namespace

Mfma2Plan mfma2_plan(const cg_conv_desc& d) {
  Mfma2Plan g{};
  g.ok = 0;
  if (d.in_dtype != CG_BF16 && d.in_dtype != CG_I8) return g;
  if (d.groups > 1 || d.tau_c > 0.0f) return g;   // channel grouping, channel-wise gate: row-tiled and plain kernels only
  if (d.kh != 3 || d.kw != 3) return g;
  g.elem_bytes = d.in_dtype == CG_BF16 ? 2 : 1;
  g.ch = 16 / g.elem_bytes;
  const int c_cond = d.c_in - d.c_base;
  const long long xps = d.x_pixel_stride ? d.x_pixel_stride : d.c_in;
  if (d.c_base % g.ch || c_cond % g.ch || xps % g.ch) return g;
  if (d.c_out % kBN) return g;
  const int ho = (d.h + 2 * d.pad - 3) / d.stride + 1, wo = (d.w + 2 * d.pad - 3) / d.stride + 1;
  // 32-bit byte offsets and 16-bit row numbers inside the kernel
  if ((long long)d.n_max * d.h * d.w * xps * g.elem_bytes >= (1ll << 31)) return g;
  if ((long long)d.n_max * ho * wo >= (1ll << 30)) return g;
  if ((long long)d.n_max * (d.h + 2 * d.pad) >= 65536 || (long long)d.n_max * ho >= 65536) return g;
  g.n_cb = d.c_out / kBN;
  g.hp = d.h + 2 * d.pad;
  g.pw = (wo - 1) * d.stride + 3;
  g.magic_hp = magic_of(g.hp);
  g.magic_ho = magic_of(ho);
  g.magic_wo = magic_of(wo);
  const bool gated = c_cond > 0;
  const int cq0 = d.c_base / g.ch, cq1 = c_cond / g.ch;

  const long long rows = (long long)d.n_max * ho;
  for (int cbq = 4; cbq >= 1; cbq >>= 1) {
    if (cq0 % cbq || (gated && cq1 % cbq)) continue;
    for (int ngw = 2; ngw >= 1; --ngw) {
      g.ngw = ngw;
      g.bm = ngw * 16 * kWaves;
      g.tr = g.bm / wo;
      if (g.tr < 1) continue;
      if (g.tr > rows) g.tr = (int)rows;
      const long long tiles = (rows + g.tr - 1) / g.tr;
      // prefer the large tile only when it still fills the 256 CUs
      if (ngw == 2 && tiles * g.n_cb < 256) continue;
      g.bm_valid = g.tr * wo;
      g.ng = (g.bm_valid + 15) / 16;
      int pr = 0;
      for (int r0 = 0; r0 < ho; ++r0) {
        const int r1 = r0 + g.tr - 1;
        const int rows_here = (r1 / ho) * g.hp + (r1 % ho) * d.stride - r0 * d.stride + 3;
        if (rows_here > pr) pr = rows_here;
      }
      g.pr_max = pr;
      g.npix = g.pr_max * g.pw;
      if (g.npix >= 65536) continue;
      g.max_imgs = (ho - 1 + g.tr - 1) / ho + 1;

      int off = 0;
      g.lds_goff = off;
      off += align_up(g.npix * 4, 16);
      g.lds_outpp = off;
      off += g.bm * 4;
      g.lds_outm = off;
      off += g.bm * 4;
      g.lds_flag = off;
      off += g.bm * 4;
      g.lds_clist = off;
      off += g.bm * 4;
      g.lds_rank = off;
      off += g.bm * 4;
      g.lds_dbits = off;
      off += g.bm * 8;
      g.lds_colcnt = off;
      off += g.max_imgs * kBN * 4;
      if (off > kTabBytes) continue;

      // plane stride: a multiple of 256 bytes for unit stride, 16 past one for stride 2 (where the
      // lanes of a group are 32 bytes apart); room for the zero pixel after the npix real ones
      g.pln = align_up((g.npix + 1) * 16, 256) + (d.stride == 2 ? 16 : 0);
      g.nps = g.pln / 16;
      g.magic_nps = magic_of(g.nps);
      g.cbq = cbq;
      g.tsteps = (9 * cbq + 3) / 4;
      g.kp = (cbq * g.nps + kThreads - 1) / kThreads;
      if (g.kp > kKP) continue;
      g.patch_bytes = align_up(cbq * g.pln, 1024);
      g.w_bytes = g.tsteps * 4 * kBN * 16;
      g.stage_bytes = g.patch_bytes + g.w_bytes;
      if (g.stage_bytes > kStageBytes) continue;
      if (g.bm * kBN * 4 > kStageBytes) continue;
      g.lds_total = 2 * kStageBytes + kTabBytes;
      g.stages[0] = cq0 / cbq;
      g.stages[1] = gated ? cq1 / cbq : 0;
      g.wpk_stage_bytes = (size_t)g.w_bytes;
      g.wpk_base_bytes = (size_t)g.n_cb * g.stages[0] * g.wpk_stage_bytes;
      g.wpk_cond_bytes = (size_t)g.n_cb * g.stages[1] * g.wpk_stage_bytes;
      g.ok = 1;
      return g;
    }
  }
  return g;
}

hipError_t launch_mfma2_pack(const Mfma2Plan& g, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s) {
  hipError_t e = launch_pack_weights(p.w_base, wpk_base, p.c_out, 9, p.c_base, g.elem_bytes, g.ch, kBN, g.cbq,
                                     g.stages[0], g.tsteps, s);
  if (e != hipSuccess) return e;
  if (g.stages[1] > 0)
    e = launch_pack_weights(p.w_cond, wpk_cond, p.c_out, 9, p.c_cond, g.elem_bytes, g.ch, kBN, g.cbq, g.stages[1],
                            g.tsteps, s);
  return e;
}

hipError_t launch_mfma2(const Mfma2Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (p.in_dtype == CG_BF16) return launch_dtype<Bf16Traits>(g, p, w0, w1, s);
  return launch_dtype<I8Traits>(g, p, w0, w1, s);
}

}  // namespace cg
