// Large-tile matrix-core kernel of the gated convolution (bf16 and int8 MFMA, 32x32 blocks).
//
// One workgroup of four wavefronts, alone on its compute unit, owns a tile of BM = 128 * FP / WN
// consecutive output pixels (whole output rows of the batch, numbered R = img*Ho + ho, possibly
// straddling images) times BN = 64 * WN output channels and runs the whole layer for them (Eq. 1
// of the channel-gating paper).  A wavefront multiplies FP 32-pixel fragments by 64 channels: with
// FP = 4 every K step costs six 16-byte operand reads for eight 32x32 MFMAs, which is what keeps
// the LDS read rate below what the matrix cores can consume.
//
//   base path   implicit GEMM over taps x base channels, taken transposed (weights are the row
//               operand, pixels the column operand; the prepacked weight rows are permuted), so a
//               lane ends up with 16 consecutive channels of one pixel per accumulator: gate and
//               output function work on registers.
//   gate        accumulators against the per-channel thresholds (merged gate, Sec. 3.2); each
//               lane packs its 32 decisions; the decision words of the tile meet in LDS and leave
//               as one coalesced store.
//   compaction  ballot / prefix sum over the tile's pixels with a fired gate lists them; 32-pixel
//               fragments of that list are dealt to the wavefronts.  Pooling the fired pixels of
//               up to 512 pixels is what lets the conditional path run on full MFMA blocks while
//               its weights are streamed once per tile.
//   cond. path  the same loop over taps x remaining channels on the listed pixels only (the pixel
//               operand is gathered from the LDS patch by per-lane address).
//   combine     R goes through an LDS tile back to the lanes that hold P; S = P + d*R, then
//               scale/shift by decision, residual, ReLU, convert (Eq. 1).
//
// K is walked in stages of CPS 16-byte channel chunks per pixel times all taps.  A stage's input
// patch ([pixel slot][CPS chunk positions], slot = patch_row * P + wi + pad with P a power of two;
// the zero padding of a row is fetched from a page of zeros) and its weight slab sit in one of NB
// LDS buffers.  The buffers are filled by LDS-direct loads issued NB - 1 stages ahead: with a
// workgroup's whole chain of stages a few microseconds long, what bounds the layer is how many
// bytes are in flight, not how fast a stage multiplies.  The loads are issued from inline assembly
// and waited for with explicit counts: the compiler, which would drain every LDS-direct load it
// knows of before the next LDS read, sees only ordinary LDS reads.
#pragma once
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "cg_mfma_common.h"
#include "tile_cfg.h"

namespace cg {

namespace tile {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(16))) int i32x16;

constexpr int kNT = 256;   // threads per workgroup: four wavefronts, one per SIMD

// 32x32 output block; lane l supplies row / column l%32 and the 16-byte K chunk l/32 of either
// operand; it receives column l%32, rows 8*(i/4) + 4*(l/32) + i%4 in register i.
struct Bf16Tile {
  using Base = Bf16Traits;
  using acc16 = f32x16;
  using acc_t = float;
  static __device__ __forceinline__ acc16 mfma(i32x4 rows, i32x4 cols, acc16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rows), __builtin_bit_cast(bf16x8, cols),
                                                   c, 0, 0, 0);
  }
};

struct I8Tile {
  using Base = I8Traits;
  using acc16 = i32x16;
  using acc_t = int32_t;
  static __device__ __forceinline__ acc16 mfma(i32x4 rows, i32x4 cols, acc16 c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(rows, cols, c, 0, 0, 0);
  }
};

__device__ __forceinline__ int bits_of(float f) { return __float_as_int(f); }
__device__ __forceinline__ int bits_of(int v) { return v; }
__device__ __forceinline__ void set_bits(int b, float& f) { f = __int_as_float(b); }
__device__ __forceinline__ void set_bits(int b, int& v) { v = b; }

// exact x / d for x, d < 65536 with magic = ceil(2^32 / d); magic 0 stands for d = 1
__device__ __forceinline__ int mdiv(int x, unsigned magic) { return magic ? (int)__umulhi((unsigned)x, magic) : x; }

template <int... I, typename F>
__device__ __forceinline__ void sfor_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void sfor(F&& f) {
  sfor_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

// Position of channel chunk q of pixel slot s inside the slot: q ^ swz(s).  Sixteen lanes read
// sixteen consecutive slots; the XOR spreads the slots that would share LDS banks (slots
// 256 / (16*CPS) apart) over different chunk positions.
template <int CPS>
__device__ __forceinline__ int swz(int slot) {
  if constexpr (CPS == 1) return 0;
  return (slot >> ilog2(16 / CPS)) & (CPS - 1);
}
template <int CPS>
__device__ __forceinline__ int slot_byte(int slot, int h) {
  if constexpr (CPS == 1) return slot * 16;
  return slot * (16 * CPS) + ((h ^ swz<CPS>(slot)) & (CPS - 1)) * 16;
}


// s_waitcnt vmcnt(n): at most n vector-memory operations of this wavefront still in flight
// (the count is a 6-bit field split over bits 3:0 and 15:14; lgkmcnt and expcnt are left open)
#define CG_TILE_VMCNT(n) (0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// for n = r * PER with 0 <= r <= MAXR
template <int MAXR, int PER>
__device__ __forceinline__ void wait_vm_stages(int r) {
  static_assert(MAXR * PER <= 63, "the wait counter has six bits");
  if constexpr (MAXR == 0) {
    __builtin_amdgcn_s_waitcnt(CG_TILE_VMCNT(0));
  } else {
    if (r >= MAXR)
      __builtin_amdgcn_s_waitcnt(CG_TILE_VMCNT(MAXR * PER));
    else
      wait_vm_stages<MAXR - 1, PER>(r);
  }
}

template <typename Tr, int TAPS, int CPS, int FP, int WN, int NB>
struct Cfg {
  static constexpr TileCfgSize Z = tile_cfg_size(TAPS, CPS, FP, WN);
  static constexpr int WM = 4 / WN;                       // wavefronts across the pixels
  static constexpr int BN = Z.bn;                         // output channels per workgroup
  static constexpr int BM = Z.bm;                         // pixels per tile
  static constexpr int SB = 16 * CPS;                     // bytes per pixel slot
  static constexpr int KS = Z.ks;                         // K steps per stage
  static constexpr int KW = Z.kw;                         // weight load instructions per wavefront per stage
  static constexpr int WBP = Z.wbp;                       // bytes of a stage's weight slab, padded to 4 KB
  static constexpr int KP = Z.kp;                         // patch load instructions per wavefront per stage
  static constexpr int PBM = Z.pbm;                       // bytes of a stage's patch, at most
  static constexpr int LPS = Z.lps;                       // load instructions per wavefront per stage
  static constexpr int SZ = Z.sz;                         // bytes per stage buffer
  static constexpr int D = NB - 1;                        // stages the loads run ahead
  static constexpr int FPR = FP >= 4 ? 2 : 1;             // listed fragments per wavefront and conditional pass
  static constexpr int CAP = 32 * WM * FPR;               // listed pixels per conditional pass
  static constexpr int WPP = BN / 32;                     // decision words per pixel
  static constexpr int RS = BN * 4 + 16;                  // bytes per row of the R tile: BN sums + 16 bytes of skew
  static constexpr int TAB = Z.tab;
  static constexpr int LDS = NB * SZ + TAB;
  static_assert(NB == Z.nb, "the buffer count follows from the sizes");
  static_assert(32 * RS <= SZ, "a 32-row slice of the R tile must fit a stage buffer");
  static_assert(4 * 32 * (64 * 2 + 16) <= SZ, "the wavefronts' output tiles must fit a stage buffer");
  static_assert(NB >= 2 && NB <= 4, "two to four stage buffers");
};

template <typename Tr, int TAPS, int CPS, int FP, int WN, int NB>
__global__ __launch_bounds__(kNT) void gated_conv_tile_kernel(Params p, TilePlan g, TileGeo q,
                                                              const char* __restrict__ wpk0,
                                                              const char* __restrict__ wpk1) {
  using C = Cfg<Tr, TAPS, CPS, FP, WN, NB>;
  using acc16 = typename Tr::acc16;
  using acc_t = typename Tr::acc_t;
  using Base = typename Tr::Base;
  constexpr int BM = C::BM, BN = C::BN, WM = C::WM, KS = C::KS, KP = C::KP, KW = C::KW, FPR = C::FPR, WPP = C::WPP;
  constexpr int D = C::D;
  constexpr int PAIRS = CPS >= 2 ? CPS / 2 : 1;

  __shared__ __align__(1024) char ring[NB * C::SZ];   // the stage buffers
  __shared__ __align__(16) char smem[C::TAB];
  char* const buf0 = ring;
  int* pslot = (int*)smem;                         // [BM] tile pixel -> patch slot of its tap (0,0)
  int* clist = pslot + BM;                         // [BM] compacted position -> patch slot
  uint32_t* bmp = (uint32_t*)(clist + BM);         // [BM][WPP] decision words of the tile
  uint16_t* rank = (uint16_t*)(bmp + WPP * BM);    // [BM] tile pixel -> compacted position
  // the eight per-channel tables of this channel block, [8][BN] words, as they lie in `packed`:
  // float layers: 0 lower threshold, 1 upper threshold, 2..5 scale0, shift0, scale1, shift1;
  // int8 layers: 0 threshold
  acc_t* tlo = (acc_t*)(rank + BM);
  acc_t* thi = tlo + BN;
  float* aff = (float*)(thi + BN);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int lj = lane & 31, lh = lane >> 5;

  // Block id mod 8 is the XCD.  Normally the blocks that share a pixel tile sit on one XCD and an
  // XCD takes a contiguous run of tiles (a tile's input and the halo rows it shares with its
  // neighbours are fetched into one L2); xcd_cb: the blocks that share a channel block sit on one
  // XCD instead, so that each L2 holds an eighth of the weights.
  int tile, cbk;
  const int total_rows = q.n * q.ho;
  {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    if (g.xcd_cb) {
      const int ncb8 = g.n_cb >> 3;
      tile = slot / ncb8;
      cbk = (slot - tile * ncb8) * 8 + xcd;
    } else {
      const int grp = slot / g.n_cb;
      cbk = slot - grp * g.n_cb;
      const int tiles = (total_rows + g.tr - 1) / g.tr;
      tile = xcd * ((tiles + 7) >> 3) + grp;
    }
  }
  const int R0 = tile * g.tr;
  if (R0 >= total_rows) return;

  const int S0 = g.stages[0];
  const int S1 = (p.gated && !p.gate_only) ? g.stages[1] : 0;
  const int eb = g.elem_bytes;

  const long long m0 = (long long)R0 * q.wo;
  const int rows_here = total_rows - R0 < g.tr ? total_rows - R0 : g.tr;
  int bmv = rows_here * q.wo;                       // output pixels of this tile
  if (m0 + bmv > q.m_valid) bmv = (int)(q.m_valid - m0);
  const int img0 = mdiv(R0, q.magic_ho);
  const int rho0 = img0 * q.hp + (R0 - img0 * q.ho) * q.stride;   // stacked padded input row of patch row 0
  const int rowb = C::SB << g.logp;                 // bytes per patch row

  // ---- this lane's share of a stage's patch: 16-byte position (wave + 4k)*64 + lane; a position
  // outside the image is fetched from the page of zeros
  const char* xbytes = (const char*)p.x;
  int voff[KP];
#pragma unroll
  for (int k = 0; k < KP; ++k) {
    voff[k] = -1;
    const int pos16 = tid + kNT * k;
    if (pos16 < g.n16) {
      const int sl = pos16 / CPS, cp = pos16 % CPS;
      const int qc = cp ^ swz<CPS>(sl);
      const int prow = sl >> g.logp, c = sl & ((1 << g.logp) - 1);
      const int rho = rho0 + prow;
      const int img = mdiv(rho, q.magic_hp);
      const int hi = rho - img * q.hp - q.pad, wi = c - q.pad;
      if (prow < g.pr && img < q.n && hi >= 0 && hi < q.h && wi >= 0 && wi < q.w) {
        const long long lin = ((long long)img * q.h + hi) * q.w + wi;
        if (lin < q.in_valid) voff[k] = (int)lin * q.xps + qc * 16;    // the plan keeps x below 2 GiB
      }
    }
  }

  // x at the first channel of stage sg (counted over both phases).  The base phase starts at this
  // block's first base channel; the conditional phase walks the channels in order and jumps over
  // the base channels (without grouping these are the first c_base; with grouping, Sec. 3.3, those
  // of the block's own group, or none when the block covers several groups and the packed weights
  // carry zeros instead).
  int base_ch0 = 0, gap_start = 0, gap_len = p.c_base;
  if (g.grp_mode == 1) {
    base_ch0 = gap_start = (cbk * BN / p.cpg) * p.c_base;
  } else if (g.grp_mode == 2) {
    base_ch0 = p.groups > 1 ? cbk * g.gsp * p.c_base : 0;
    gap_len = 0;
  }
  auto x_src = [&](int sg) __attribute__((always_inline)) {
    const int ph = sg >= S0 ? 1 : 0;
    const int ss = ph ? sg - S0 : sg;
    int chn = ss * CPS * g.ch;
    chn = ph ? (chn >= gap_start ? chn + gap_len : chn) : base_ch0 + chn;
    return xbytes + (long long)chn * eb;
  };
  const char* const wbase0 = wpk0 + (size_t)cbk * g.stages[0] * C::WBP + tid * 16;
  const char* const wcond0 = wpk1 + (size_t)cbk * g.stages[1] * C::WBP + tid * 16;
  const char* const zeros = (const char*)p.zeros;

  // the LDS-direct loads of stage sg into buffer b: every wavefront issues KW + KP instructions of
  // 1 KB each (lane l's 16 bytes land at the given LDS address + 16*l), whatever its lanes fetch,
  // so that the wait counts below are compile-time values
  auto dma16 = [&](const char* src, char* dst) __attribute__((always_inline)) {
    const unsigned la = (unsigned)(uintptr_t)dst;     // low half of a generic LDS address = LDS byte offset
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(la), "v"(src) : "memory");
  };
  // the per-channel tables come first, as 4-byte LDS-direct loads (256 bytes an instruction): table
  // t of `packed` starts at thr_f + t * table_stride; the loads are older than every stage's, so the
  // first stage's wait covers them
  {
    constexpr int NTI = 8 * BN / 64;          // instructions for the whole block of tables
#pragma unroll
    for (int k = 0; k < NTI / 4; ++k) {
      const int i = wave + 4 * k;             // instruction: table i / (BN/64), 64-channel part i % (BN/64)
      const int t = i / (BN / 64), part = i % (BN / 64);
      const char* src = (const char*)p.thr_f + (size_t)t * p.table_stride + ((size_t)cbk * BN + part * 64 + lane) * 4;
      const unsigned la = (unsigned)(uintptr_t)((char*)tlo + (t * BN + part * 64) * 4);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(la), "v"(src) : "memory");
    }
  }
  auto issue_part = [&](int b, int sg, auto part_tag, auto parts_tag) __attribute__((always_inline)) {
    // slice `part` of `parts` of a stage's load instructions
    constexpr int part = decltype(part_tag)::value, parts = decltype(parts_tag)::value;
    constexpr int lo = part * C::LPS / parts, hi = (part + 1) * C::LPS / parts;
    if constexpr (lo < hi) {
      char* dst = ring + b * C::SZ + wave * 1024;
      const char* xs = x_src(sg);
      const char* ws = sg >= S0 ? wcond0 + (size_t)(sg - S0) * C::WBP : wbase0 + (size_t)sg * C::WBP;
#pragma unroll
      for (int i = lo; i < hi; ++i) {
        if (i < KW) {
          dma16(ws + i * 4096, dst + C::PBM + i * 4096);
        } else {
          const int k = i - KW;
          dma16(voff[k] >= 0 ? xs + voff[k] : zeros, dst + k * 4096);
        }
      }
    }
  };
  auto issue = [&](int b, int sg) __attribute__((always_inline)) {
    char* dst = ring + b * C::SZ + wave * 1024;
    const char* xs = x_src(sg);
    const char* ws = sg >= S0 ? wcond0 + (size_t)(sg - S0) * C::WBP : wbase0 + (size_t)sg * C::WBP;
#pragma unroll
    for (int k = 0; k < KW; ++k) dma16(ws + k * 4096, dst + C::PBM + k * 4096);
#pragma unroll
    for (int k = 0; k < KP; ++k) dma16(voff[k] >= 0 ? xs + voff[k] : zeros, dst + k * 4096);
  };
  // barrier between LDS writers and readers without __syncthreads()'s drain of every load in flight
  auto lds_barrier = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): this wavefront's LDS accesses are done
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // ---- this lane's base-path pixels ------------------------------------------------------------
  constexpr int NTC = TAPS == 9 ? 3 : 1;     // tap columns
  int pix[FP];
  bool pval[FP];
  int pa[FP][NTC];       // patch byte offsets of the tap columns, kernel row 0
#pragma unroll
  for (int fp = 0; fp < FP; ++fp) {
    pix[fp] = (wm * FP + fp) * 32 + lj;
    pval[fp] = pix[fp] < bmv;
    const int i = pval[fp] ? pix[fp] : 0;            // fragments past the tile's end read pixel 0 and are dropped
    const int lr = mdiv(i, q.magic_wo), wo_ = i - lr * q.wo;
    const int R = R0 + lr;
    const int img = mdiv(R, q.magic_ho), hq = R - img * q.ho;
    const int slot = ((img * q.hp + hq * q.stride - rho0) << g.logp) + wo_ * q.stride;
    if (lh == 0 && wn == 0) pslot[pix[fp]] = slot;
#pragma unroll
    for (int c = 0; c < NTC; ++c) pa[fp][c] = slot_byte<CPS>(slot + c, lh);
  }
  // CPS = 1 pairs the chunks of two taps in one K step: lane half h of step k takes tap 2k + h
  // (the ninth tap's partner is a zero weight and re-reads the ninth tap)
  int tofs[CPS == 1 ? KS : 1];
  if constexpr (CPS == 1) {
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      int t = 2 * k + lh;
      t = t < TAPS ? t : TAPS - 1;
      tofs[k] = TAPS == 9 ? (t / 3) * rowb + (t % 3) * 16 : 0;
    }
  } else {
    tofs[0] = 0;
  }
  for (int i = tid; i < WPP * BM; i += kNT) bmp[i] = 0u;

  acc16 accP[FP][2], accR[FPR][2];
#pragma unroll
  for (int fp = 0; fp < FP; ++fp)
#pragma unroll
    for (int fl = 0; fl < 2; ++fl)
#pragma unroll
      for (int i = 0; i < 16; ++i) accP[fp][fl][i] = 0;
#pragma unroll
  for (int k = 0; k < FPR; ++k)
#pragma unroll
    for (int fl = 0; fl < 2; ++fl)
#pragma unroll
      for (int i = 0; i < 16; ++i) accR[k][fl][i] = 0;

  const int wofs = C::PBM + lh * (16 * BN) + (wn * 64 + lj) * 16;   // lane's offset of its weight rows of K step 0

  // One stage for NL pixel fragments out of a stage buffer.  Operands of two K steps are in
  // registers: the reads of step k+1 go out before the MFMAs of step k; the scheduling barriers
  // keep the compiler from hoisting every read of the stage to its top.
  auto mma_stage = [&](auto nl_tag, auto& acc, const auto& base, const char* sb, auto&& iss)
                       __attribute__((always_inline)) {
    constexpr int NL = decltype(nl_tag)::value;
    if constexpr (NL == 0) {
      sfor<KS>([&](auto kc) __attribute__((always_inline)) { iss(kc); });
    } else {
      const char* pat = sb;
      const char* wl = sb + wofs;
      i32x4 a[2][2], bb[2][NL];
      auto read_step = [&](auto kc) __attribute__((always_inline)) {
        constexpr int ks = decltype(kc)::value;
        constexpr int n = ks & 1;
        a[n][0] = *(const i32x4*)(wl + ks * 32 * BN);
        a[n][1] = *(const i32x4*)(wl + ks * 32 * BN + 512);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          int ad;
          if constexpr (CPS == 1) {
            ad = base[i][0] + tofs[ks];
          } else {
            constexpr int tap = (2 * ks) / CPS, j = ks % PAIRS;
            constexpr int r = TAPS == 9 ? tap / 3 : 0, c = TAPS == 9 ? tap % 3 : 0;
            ad = (base[i][c] + r * rowb) ^ (j * 32);
          }
          bb[n][i] = *(const i32x4*)(pat + ad);
        }
      };
      read_step(std::integral_constant<int, 0>{});
      sfor<KS>([&](auto kc) __attribute__((always_inline)) {
        constexpr int ks = decltype(kc)::value;
        constexpr int n = ks & 1;
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (ks + 1 < KS) read_step(std::integral_constant<int, ks + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        acc[0][0] = Tr::mfma(a[n][0], bb[n][0], acc[0][0]);
        __builtin_amdgcn_sched_barrier(0);
        iss(kc);          // a slice of the next loads goes out behind the first MFMA of the K step
        __builtin_amdgcn_sched_barrier(0);
        acc[0][1] = Tr::mfma(a[n][1], bb[n][0], acc[0][1]);
#pragma unroll
        for (int i = 1; i < NL; ++i) {
          acc[i][0] = Tr::mfma(a[n][0], bb[n][i], acc[i][0]);
          acc[i][1] = Tr::mfma(a[n][1], bb[n][i], acc[i][1]);
        }
      });
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  unsigned dlane[FP];   // this lane's decisions of pixel fp: bit 16*fl + i = channel 64*wn + 32*fl + 16*lh + i
#pragma unroll
  for (int fp = 0; fp < FP; ++fp) dlane[fp] = 0u;
  int n_act = 0;        // fired pixels of the tile
  int nl = 0;           // listed fragments of this wavefront in the current conditional pass
  int pac[FPR][NTC];    // patch offsets of this lane's listed pixels
#pragma unroll
  for (int k = 0; k < FPR; ++k)
#pragma unroll
    for (int c = 0; c < NTC; ++c) pac[k][c] = 0;

  // the listed fragments of a conditional pass: fragment c = k*WM + wm of the pass goes to slot k
  auto deal = [&](int pass0) __attribute__((always_inline)) {
    const int left = n_act - pass0;
    const int nfrag = (left + 31) >> 5;
    int n = 0;
#pragma unroll
    for (int k = 0; k < FPR; ++k) {
      const int c = k * WM + wm;
      if (c < nfrag) n = k + 1;
      const int li = pass0 + c * 32 + lj;
      const int slot = clist[li < n_act ? li : pass0];
#pragma unroll
      for (int cc = 0; cc < NTC; ++cc) pac[k][cc] = slot_byte<CPS>(slot + cc, lh);
#pragma unroll
      for (int fl = 0; fl < 2; ++fl)
#pragma unroll
        for (int i = 0; i < 16; ++i) accR[k][fl][i] = 0;
    }
    nl = __builtin_amdgcn_readfirstlane(n);
  };

  // ---- gate, decision words, compaction (runs once, when the base path is complete) ----------------
  auto gate_and_compact = [&]() __attribute__((always_inline)) {
    // the accumulators are read right after the MFMAs; their results need the wait states
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    uint16_t* bmph = (uint16_t*)bmp;
#pragma unroll
    for (int fp = 0; fp < FP; ++fp) {
      unsigned dl = 0u;
#pragma unroll
      for (int fl = 0; fl < 2; ++fl) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int c0 = 64 * wn + 32 * fl + 16 * lh + 4 * q4;
          const i32x4 lo4 = *(const i32x4*)(tlo + c0);
          const i32x4 hi4 = *(const i32x4*)(thi + c0);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const acc_t v = accP[fp][fl][4 * q4 + e];
            bool f;
            if constexpr (Base::kDtype == CG_I8)
              f = Base::fires(v, lo4[e], hi4[e]);
            else
              f = Base::fires(v, __int_as_float(lo4[e]), __int_as_float(hi4[e]));
            dl |= (f ? 1u : 0u) << (16 * fl + 4 * q4 + e);
          }
        }
      }
      if (!pval[fp]) dl = 0u;
      if (p.chan_mask) {
        // channel-wise gate (Sec. 3.2): only the channels that keep their conditional path in this image
        const int img = (int)((m0 + (pval[fp] ? pix[fp] : 0)) / ((long long)p.ho * p.wo));
        const uint32_t* mw = p.chan_mask + (long long)img * p.words + cbk * WPP + wn * 2;
        dl &= ((mw[0] >> (16 * lh)) & 0xffffu) | (((mw[1] >> (16 * lh)) & 0xffffu) << 16);
      }
      dlane[fp] = dl;
      bmph[pix[fp] * (2 * WPP) + wn * 4 + lh] = (uint16_t)(dl & 0xffffu);
      bmph[pix[fp] * (2 * WPP) + wn * 4 + 2 + lh] = (uint16_t)(dl >> 16);
    }
    lds_barrier();
    // (the decision words leave for memory after the last stage: a store between the loads in flight
    // would make their completion order unknown to the counted waits)
    // every wavefront scans all pixels; wavefront w places the 64-pixel groups w, w + 4, ...
    int run = 0;
#pragma unroll
    for (int c = 0; c < BM / 64; ++c) {
      const int px = c * 64 + lane;
      uint32_t any = 0u;
#pragma unroll
      for (int w = 0; w < WPP; ++w) any |= bmp[px * WPP + w];
      const unsigned long long bal = __ballot(any != 0u);
      if ((c & 3) == wave && ((bal >> lane) & 1ull)) {
        const int idx = run + __popcll(bal & ((1ull << lane) - 1ull));
        clist[idx] = pslot[px];
        rank[px] = (uint16_t)idx;
      }
      run += __popcll(bal);
    }
    n_act = run;
    lds_barrier();
  };

  // ---- combine: R (the pass's compacted rows) goes through LDS to the lanes that hold P; the
  // conditional sum is dropped where that channel did not fire (Eq. 1).  No load is in flight and
  // the stage buffers are free: the whole R tile of the pass lies in them at once.
  auto combine = [&](int pass0) __attribute__((always_inline)) {
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    constexpr int RS = C::RS;
    static_assert(C::CAP * RS <= NB * C::SZ, "the R tile of a pass must fit the stage buffers");
#pragma unroll
    for (int k = 0; k < FPR; ++k) {
      if (k < nl) {
        char* row = ring + ((k * WM + wm) * 32 + lj) * RS + (wn * 64 + lh * 16) * 4;
#pragma unroll
        for (int fl = 0; fl < 2; ++fl)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            i32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const acc_t rv = accR[k][fl][4 * q4 + e];
              v[e] = bits_of(rv);
            }
            *(i32x4*)(row + fl * 128 + q4 * 16) = v;
          }
      }
    }
    __syncthreads();
#pragma unroll
    for (int fp = 0; fp < FP; ++fp) {
      // a pixel without a row in this pass adds nothing; a fragment with no such pixel is skipped
      const int r = (int)rank[pix[fp]] - pass0;
      const bool ok = dlane[fp] != 0u && r >= 0 && r < C::CAP;
      if (__ballot(ok) != 0ull) {
        const unsigned dm = ok ? dlane[fp] : 0u;
        const char* row = ring + (ok ? r : 0) * RS + (wn * 64 + lh * 16) * 4;
#pragma unroll
        for (int fl = 0; fl < 2; ++fl)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const i32x4 v = *(const i32x4*)(row + fl * 128 + q4 * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const bool on = (dm >> (16 * fl + 4 * q4 + e)) & 1u;
              acc_t rv;
              set_bits(v[e], rv);
              accP[fp][fl][4 * q4 + e] += on ? rv : (acc_t)0;
            }
          }
      }
    }
    __syncthreads();
  };

  // ---- the stage pipeline ---------------------------------------------------------------------------
  // Pass 0 walks the base stages, takes the gate, and walks the conditional stages on the first CAP
  // listed pixels; a tile with more fired pixels repeats the conditional stages for the next CAP
  // (rare: more than half of the tile fired).  Step u of a pass uses buffer u % NB.
  for (int pass = 0;; ++pass) {
    const int soff = pass ? S0 : 0;
    int T = pass ? S1 : S0 + S1;
#pragma unroll
    for (int b = 0; b < D; ++b)
      if (b < T) issue(b, soff + b);
    int b = 0;               // buffer of step u = u % NB
#pragma nounroll
    for (int u = 0; u < T; ++u) {
      // this wavefront's part of stage u has landed once at most the loads of the later stages are
      // in flight; after the barrier everybody's part has, and buffer (u - 1) % NB is free
      const int later = T - 1 - u < D - 1 ? T - 1 - u : D - 1;
      wait_vm_stages<D - 1, C::LPS>(later);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const bool more = u + D < T;
      const int bn_ = b == 0 ? NB - 1 : b - 1, sgn = soff + u + D;
      auto iss = [&](auto kc) __attribute__((always_inline)) {
        if (more) issue_part(bn_, sgn, kc, std::integral_constant<int, KS>{});
      };
      const char* sb = ring + b * C::SZ;
      const int sg = soff + u;
      if (sg < S0) {
        mma_stage(std::integral_constant<int, FP>{}, accP, pa, sb, iss);
      } else {
        if (pass == 0 && sg == S0) {
          gate_and_compact();
          if (n_act == 0) T = 0;          // nothing fired: the conditional stages are dropped
          deal(0);
        }
        if (u < T) {
          if (nl == FPR)
            mma_stage(std::integral_constant<int, FPR>{}, accR, pac, sb, iss);
          else if (FPR == 2 && nl == 1)
            mma_stage(std::integral_constant<int, 1>{}, accR, pac, sb, iss);
          else
            mma_stage(std::integral_constant<int, 0>{}, accR, pac, sb, iss);
        }
      }
      b = b + 1 == NB ? 0 : b + 1;
    }
    if (!p.gated) break;
    if (pass == 0 && S1 == 0) {
      gate_and_compact();                     // a gate-only pass stops after the base stages
      break;
    }
    // drain what the dropped stages left in flight; every wavefront is done with the buffers
    __builtin_amdgcn_s_waitcnt(CG_TILE_VMCNT(0));
    __syncthreads();
    if (n_act == 0) break;
    combine(pass * C::CAP);
    if ((pass + 1) * C::CAP >= n_act) break;
    deal((pass + 1) * C::CAP);
  }
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
  __builtin_amdgcn_s_waitcnt(CG_TILE_VMCNT(0));
  __syncthreads();
  if (p.gated && p.bitmap) {
    for (int i = tid; i < bmv * WPP; i += kNT) {
      const int px = i / WPP, w = i % WPP;
      p.bitmap[(m0 + px) * p.words + cbk * WPP + w] = bmp[i];
    }
  }
  if (p.gate_only) return;   // first pass of the channel-wise gate: the decisions are all it produces

  // ---- output function on 16 consecutive channels per accumulator ---------------------------------
  const int ob = p.out_dtype == CG_BF16 ? 2 : p.out_dtype == CG_I8 ? 1 : 4;
  const int cb0 = cbk * BN + 64 * wn;       // first channel of this wavefront
  if (p.shuffle) {
    // shuffled channel order (Sec. 3.3): channel j of group i goes to position j*groups + i of its
    // pixel, one element at a time
#pragma unroll
    for (int fp = 0; fp < FP; ++fp) {
      if (!pval[fp]) continue;
#pragma unroll
      for (int fl = 0; fl < 2; ++fl) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int co = cb0 + 32 * fl + 16 * lh + i;
          const int grp = co / p.cpg;
          const long long o = (m0 + pix[fp]) * p.c_out + (co - grp * p.cpg) * p.groups + grp;
          const bool fired = p.gated ? ((dlane[fp] >> (16 * fl + i)) & 1u) != 0u : true;
          const acc_t sv = accP[fp][fl][i];
          if constexpr (Base::kDtype == CG_I8) {
            store_int(p, o, finish_int(p, sv, fired, co, o));
          } else {
            store_float(p, o, finish_float(p, sv, fired, co, o));
          }
        }
      }
    }
  } else if (ob == 4) {
    // 4-byte outputs: a lane's 16 channels are 64 contiguous bytes; stored directly
#pragma unroll
    for (int fp = 0; fp < FP; ++fp) {
      if (!pval[fp]) continue;
#pragma unroll
      for (int fl = 0; fl < 2; ++fl) {
        const int co0 = cb0 + 32 * fl + 16 * lh;
        const long long o = (m0 + pix[fp]) * p.c_out + co0;
        i32x4 v[4];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const acc_t sv = accP[fp][fl][4 * q4 + e];
            v[q4][e] = bits_of(sv);
          }
        const unsigned d16 = (dlane[fp] >> (16 * fl)) & 0xffffu;
        finish_store8<Base>(p, v[0], v[1], d16 & 0xffu, co0, o);
        finish_store8<Base>(p, v[2], v[3], d16 >> 8, co0 + 8, o + 8);
      }
    }
  } else {
    // 2- and 1-byte outputs: a wavefront's 64 channels of a pixel form one row of its own LDS tile
    // (32 rows per fragment), which leaves as whole rows; only the wavefront itself touches its tile
    const int rb = 64 * ob;             // bytes per row: 128 or 64
    const int rs = rb + 16;             // skewed row stride in LDS
    const bool lean = Base::kDtype != CG_I8 && p.out_dtype == CG_BF16 &&
                      !(p.epilogue & (CG_EPI_AFFINE | CG_EPI_RESIDUAL));
    const bool fastaff = Base::kDtype != CG_I8 && p.out_dtype == CG_BF16 && (p.epilogue & CG_EPI_AFFINE);
    const float relu_lo = (p.epilogue & CG_EPI_RELU) ? 0.0f : -__builtin_inff();
    char* const wtile = buf0 + wave * (32 * (64 * 2 + 16));
#pragma unroll
    for (int fp = 0; fp < FP; ++fp) {
      {
        char* row = wtile + lj * rs;
#pragma unroll
        for (int fl = 0; fl < 2; ++fl) {
          const int cw = 32 * fl + 16 * lh;             // first of this lane's 16 channels in the wavefront's 64
          const int cl = 64 * wn + cw;                  // ... in the block
          const int co0 = cbk * BN + cl;
          const long long o = (m0 + pix[fp]) * p.c_out + co0;
          i32x4 v[4];
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const acc_t sv = accP[fp][fl][4 * q4 + e];
              v[q4][e] = bits_of(sv);
            }
          const unsigned d16 = (dlane[fp] >> (16 * fl)) & 0xffffu;
          i32x4 o0 = {0, 0, 0, 0}, o1, o2 = {0, 0, 0, 0}, o3;
          if (lean) {
            // bf16 output, no scale/shift, no residual: ReLU (or nothing) and the conversion
            if constexpr (Base::kDtype != CG_I8) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                o0[e] = (int)((uint32_t)float_to_bf16(fmaxf(__int_as_float(v[e >> 1][2 * (e & 1)]), relu_lo)) |
                              ((uint32_t)float_to_bf16(fmaxf(__int_as_float(v[e >> 1][2 * (e & 1) + 1]), relu_lo)) << 16));
                o2[e] = (int)((uint32_t)float_to_bf16(fmaxf(__int_as_float(v[2 + (e >> 1)][2 * (e & 1)]), relu_lo)) |
                              ((uint32_t)float_to_bf16(fmaxf(__int_as_float(v[2 + (e >> 1)][2 * (e & 1) + 1]), relu_lo)) << 16));
              }
            }
          } else if (fastaff) {
            // bf16 output with scale/shift by decision (tables in LDS), optional residual and ReLU
            if constexpr (Base::kDtype != CG_I8) {
              uint16_t res[16];
#pragma unroll
              for (int i = 0; i < 16; ++i) res[i] = 0;
              if ((p.epilogue & CG_EPI_RESIDUAL) && pval[fp]) {
                *(i32x4*)(res) = *(const i32x4*)((const uint16_t*)p.residual + o);
                *(i32x4*)(res + 8) = *(const i32x4*)((const uint16_t*)p.residual + o + 8);
              }
              float r16[16];
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 a0 = *(const f32x4*)(aff + cl + 4 * q4), b0 = *(const f32x4*)(aff + BN + cl + 4 * q4);
                const f32x4 a1 = *(const f32x4*)(aff + 2 * BN + cl + 4 * q4), b1 = *(const f32x4*)(aff + 3 * BN + cl + 4 * q4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int i = 4 * q4 + e;
                  const float sv = __int_as_float(v[q4][e]);
                  const bool f = p.gated ? ((d16 >> i) & 1u) != 0u : true;
                  float a = f ? fmaf(a1[e], sv, b1[e]) : fmaf(a0[e], sv, b0[e]);
                  if (p.epilogue & CG_EPI_RESIDUAL) a += bf16_to_float(res[i]);
                  r16[i] = fmaxf(a, relu_lo);
                }
              }
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                o0[e] = (int)((uint32_t)float_to_bf16(r16[2 * e]) | ((uint32_t)float_to_bf16(r16[2 * e + 1]) << 16));
                o2[e] = (int)((uint32_t)float_to_bf16(r16[8 + 2 * e]) | ((uint32_t)float_to_bf16(r16[8 + 2 * e + 1]) << 16));
              }
            }
          } else if (pval[fp]) {
            finish8<Base>(p, v[0], v[1], d16 & 0xffu, co0, o, o0, o1);
            finish8<Base>(p, v[2], v[3], d16 >> 8, co0 + 8, o + 8, o2, o3);
          }
          if (ob == 2) {
            *(i32x4*)(row + cw * 2) = o0;
            *(i32x4*)(row + cw * 2 + 16) = o2;
          } else {
            *(i32x4*)(row + cw) = i32x4{o0[0], o0[1], o2[0], o2[1]};
          }
        }
      }
      // the wavefront's LDS accesses complete in order: its rows are readable without a barrier
      __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
      asm volatile("" ::: "memory");
      __builtin_amdgcn_wave_barrier();
      // 16-byte pieces: piece id = row * (rb/16) + part
      const int ppr = rb >> 4;            // pieces per row: 8 or 4
      const int lpp = ppr == 8 ? 3 : 2;
      for (int id = lane; id < 32 * ppr; id += 64) {
        const int row = id >> lpp, part = id & (ppr - 1);
        const int px = (wm * FP + fp) * 32 + row;       // tile pixel of this row
        if (px < bmv) {
          const i32x4 v = *(const i32x4*)(wtile + row * rs + part * 16);
          *(i32x4*)((char*)p.y + ((m0 + px) * p.c_out + cbk * BN + 64 * wn) * ob + part * 16) = v;
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
      asm volatile("" ::: "memory");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <typename Tr, int TAPS, int CPS, int FP, int WN, int NB>
hipError_t launch_tile_one(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                           hipStream_t s) {
  using C = Cfg<Tr, TAPS, CPS, FP, WN, NB>;
  const long long rows = (long long)q.n * q.ho;
  const long long tiles = (rows + g.tr - 1) / g.tr;
  const long long blocks = g.xcd_cb ? tiles * g.n_cb : ((tiles + 7) / 8) * 8 * g.n_cb;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  // plan and kernel must agree
  if ((size_t)C::LDS != g.lds_bytes || C::PBM < g.n16 * 16 || NB != g.nb) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gated_conv_tile_kernel<Tr, TAPS, CPS, FP, WN, NB>), dim3((unsigned)blocks), dim3(kNT), 0, s, p,
                     g, q, (const char*)w0, (const char*)w1);
  return hipGetLastError();
}

}  // namespace tile
}  // namespace cg
