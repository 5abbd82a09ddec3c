// Row-tiled matrix-core kernel of the gated convolution (bf16 and int8 MFMA, 32x32 blocks).
//
// One workgroup of four or eight wavefronts owns a tile of 128 or 256 consecutive output pixels
// (whole output rows of the batch, numbered R = img*Ho + ho, possibly straddling images) times 64
// output channels and runs the whole layer for them (Eq. 1 of the channel-gating paper).  A
// wavefront multiplies NF 32-pixel fragments by the block's 64 channels; in the channel-split form
// (NC = 1) two wavefronts share a fragment with 32 channels each; in the loader form (LDW = 4) four
// extra wavefronts only issue the loads.  Two workgroups share a CU where LDS allows.
//
//   base path   implicit GEMM over taps x base channels.  Each wavefront owns NF 32-pixel
//               fragments x 64 channels.  The product is taken transposed (weights as the row
//               operand, pixels as the column operand), which leaves every lane with 16
//               consecutive channels of one pixel per accumulator: gate and output function
//               work on registers.
//   gate        accumulators against the per-channel thresholds (merged gate, Sec. 3.2); each
//               lane packs its 32 decisions; the decision words of the tile meet in LDS and leave
//               as one coalesced store.
//   compaction  ballot / prefix sum over the pixels with a fired gate lists them; 32-pixel
//               fragments of that list are dealt to the wavefronts.
//   cond. path  the same MFMA loop over taps x remaining channels on the listed pixels only
//               (the pixel operand is gathered from the LDS patch by per-lane address).
//   combine     R goes through a small LDS tile back to the lanes that hold P; S = P + d*R, then
//               scale/shift by decision, residual, ReLU, convert (Eq. 1); 2-byte and 1-byte
//               outputs are transposed through LDS so that every store covers whole pixel rows.
//
// Global -> LDS traffic is the scarce resource (one cache line per clock per CU, whatever part of
// the line is used), so the input patch is fetched CPS 16-byte channel chunks per pixel at a time
// (CPS = 4: 64 contiguous bytes per pixel and load-instruction quad), one "super-stage" of K, and
// kept in LDS as [pixel slot][CPS chunk positions]; chunk q of slot s sits at position q ^ f(s),
// f(s) = (s >> 2) & 3 (CPS = 4) or (s >> 3) & 1 (CPS = 2), which makes the 16-lane operand reads
// conflict-free.  Slot = patch_row * P + c with P a power of two >= max(16, W + pad) and
// c = wi + pad, so the zero padding left and right of a row are the never-loaded slots between
// rows; rows outside the image are zeroed once.  Weights stream through a two-deep ring of granules,
// one kernel row (three taps) of the super-stage each; the next granule's fetch and a part of the
// next super-stage's patch go out as LDS-direct loads while a granule is multiplied, and the wait at
// the granule's end covers only what the next granule needs (the loads of a wavefront complete in
// order).
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "cg_mfma_common.h"

namespace cg {

namespace {

constexpr int kBn = 64;                      // output channels per workgroup
constexpr int kRs = 272;                     // bytes per row of the R tile: 64 sums + 16 bytes of skew

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(16))) int i32x16;

// 32x32 output block; lane l supplies row / column l%32 and the 16-byte K chunk l/32 of either
// operand; it receives column l%32, rows 8*(i/4) + 4*(l/32) + i%4 in register i.
struct Bf16Rows {
  using Base = Bf16Traits;
  using acc16 = f32x16;
  using acc_t = float;
  static __device__ __forceinline__ acc16 mfma(i32x4 rows, i32x4 cols, acc16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rows), __builtin_bit_cast(bf16x8, cols),
                                                   c, 0, 0, 0);
  }
};

struct I8Rows {
  using Base = I8Traits;
  using acc16 = i32x16;
  using acc_t = int32_t;
  static __device__ __forceinline__ acc16 mfma(i32x4 rows, i32x4 cols, acc16 c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(rows, cols, c, 0, 0, 0);
  }
};

// bit patterns of accumulator elements (a bit cast applied directly to an element of a vector
// register array reads element 0 with this compiler, so the value is copied to a scalar first)
__device__ __forceinline__ int as_bits(float f) { return __float_as_int(f); }
__device__ __forceinline__ int as_bits(int v) { return v; }
__device__ __forceinline__ void from_bits(int b, float& f) { f = __int_as_float(b); }
__device__ __forceinline__ void from_bits(int b, int& v) { v = b; }

// exact x / d for x, d < 65536 with magic = ceil(2^32 / d); magic 0 stands for d = 1 (2^32 does not fit)
__device__ __forceinline__ int fdiv3(int x, unsigned magic) { return magic ? (int)__umulhi((unsigned)x, magic) : x; }

__device__ __forceinline__ void lds_direct16(const char* gsrc, char* ldst) {
  // each active lane copies 16 bytes from its own global address to ldst + lane*16
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)ldst, 16, 0, 0);
}

// 16-byte LDS read the compiler does not see as a memory access: it then neither orders it against
// the LDS-direct loads in flight nor waits for it; the caller waits (lgkmcnt) before using the value
__device__ __forceinline__ i32x4 lds_read16(const char* p) {
  i32x4 v;
  const unsigned addr = (unsigned)(uintptr_t)p;     // low half of a generic LDS address = LDS byte offset
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
// the same with a compile-time byte offset in the instruction (no address arithmetic per read)
template <int OFS>
__device__ __forceinline__ i32x4 lds_read16_at(unsigned addr) {
  static_assert(OFS >= 0 && OFS < 65536, "16-bit offset field");
  i32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFS) : "memory");
  return v;
}

// s_waitcnt vmcnt(n): at most n vector-memory operations of this wavefront still in flight
// (the count is a 6-bit field split over bits 3:0 and 15:14; lgkmcnt and expcnt are left open)
#define CG_VMCNT(n) (0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// for 0 <= n <= MAXN with MAXN small: a ladder of at most MAXN compares
template <int MAXN>
__device__ __forceinline__ void wait_vm_upto(int n) {
  if constexpr (MAXN == 0) {
    __builtin_amdgcn_s_waitcnt(CG_VMCNT(0));
  } else {
    if (n >= MAXN)
      __builtin_amdgcn_s_waitcnt(CG_VMCNT(MAXN));
    else
      wait_vm_upto<MAXN - 1>(n);
  }
}

// byte offset of chunk position (h ^ f(slot)) of pixel slot `slot`: the chunk lane half h multiplies
// in the first chunk pair of a super-stage; the second pair (CPS = 4) is 32 bytes away by XOR
template <int CPS>
__device__ __forceinline__ int slot_addr(int slot, int h) {
  if constexpr (CPS == 4) return slot * 64 + ((h ^ (slot >> 2)) & 3) * 16;
  return slot * 32 + ((h ^ (slot >> 3)) & 1) * 16;
}

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N-1>)
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// One weight granule of MFMAs for this wavefront: NL pixel fragments x NC 32-channel fragments (wofs
// selects the first one),
// GK = 3*CPS/2 K steps (three taps of one kernel row x CPS/2 chunk pairs).  ar[fp][c] is the lane's
// patch byte offset of fragment fp at tap column c in this kernel row; wofs the lane's offset of
// its weight rows.  The operand reads of step k+1 and a slice of the prefetch (issue(k)) are
// interleaved with the MFMAs of step k; the scheduling barriers pin that order.
template <typename Tr, int NL, int NFM, int CPS, int NC, int PD, typename IssueFn>
__device__ __forceinline__ void mma_granule(const char* __restrict__ pat, const char* __restrict__ wg, int wofs,
                                            const int (&ar)[NFM][3], typename Tr::acc16 (&acc)[NFM][NC],
                                            IssueFn&& issue) {
  constexpr int GK = 3 * CPS / 2;
  constexpr int PAIRS = CPS / 2;
  constexpr int M = NL * NC;  // MFMAs per K step
  constexpr int NR = NC + NL; // operand reads per K step
  constexpr int NB = PD + 1;  // operand register sets
  static_assert(PD >= 1 && PD * NR <= 15, "the wait counter has four bits");
  // Operands of PD + 1 K steps in registers: the reads of step k+PD go out before the MFMAs of step
  // k, so each read has PD steps to land.  LDS reads return in order, which lets the wait before
  // step k leave the reads of the later steps in flight.
  i32x4 a[NB][NC], b[NB][NL > 0 ? NL : 1];
  // the weight operands sit at compile-time offsets from one per-lane address
  const unsigned wa = (unsigned)(uintptr_t)(wg + wofs);
  auto read_step = [&](auto kc) __attribute__((always_inline)) {
    constexpr int k = decltype(kc)::value;
    constexpr int n = k % NB;
    a[n][0] = lds_read16_at<k * 2048>(wa);
    if constexpr (NC == 2) a[n][1] = lds_read16_at<k * 2048 + 512>(wa);
#pragma unroll
    for (int i = 0; i < NL; ++i) b[n][i] = lds_read16(pat + (ar[i][k / PAIRS] ^ ((k % PAIRS) * 32)));
  };
  if constexpr (NL > 0) {
    static_for<(PD < GK ? PD : GK)>([&](auto kc) __attribute__((always_inline)) { read_step(kc); });
  }
  static_for<GK>([&](auto kc) __attribute__((always_inline)) {
    constexpr int k = decltype(kc)::value;
    if constexpr (NL == 0) {
      issue(k);
    } else {
      constexpr int c = k % NB;
      // operands of step k are in registers once at most the reads of steps k+1 .. k+PD-1 are out
      constexpr int later = (GK - 1 - k) < (PD - 1) ? (GK - 1 - k) : (PD - 1);
      __builtin_amdgcn_s_waitcnt(0xC07F | ((later * NR) << 8));
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (k + PD < GK) read_step(std::integral_constant<int, k + PD>{});
      __builtin_amdgcn_sched_barrier(0);
      acc[0][0] = Tr::mfma(a[c][0], b[c][0], acc[0][0]);
      __builtin_amdgcn_sched_barrier(0);
      issue(k);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 1; j < M; ++j) acc[j / NC][j % NC] = Tr::mfma(a[c][j % NC], b[c][j / NC], acc[j / NC][j % NC]);
      __builtin_amdgcn_sched_barrier(0);
    }
  });
  if constexpr (NL > 0) {
    // The accumulators may be read right after this loop, across the branch of the last issue();
    // the compiler's count of wait states between an MFMA and a read of its result follows the
    // fall-through path only, so the required distance is put here explicitly.
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <typename Tr, int NF, int CPS, int PKB, int NWV, int NC, int LDW>
__global__ __launch_bounds__(NWV * 64, 2) void gated_conv_rows_kernel(
    Params p, Mfma3Plan g, const char* __restrict__ wpk0, const char* __restrict__ wpk1) {
  using acc16 = typename Tr::acc16;
  using acc_t = typename Tr::acc_t;
  using Base = typename Tr::Base;
  constexpr int NT = NWV * 64;                 // threads
  constexpr int RD = 2;                        // weight granules in the ring: the one in use and the next
  constexpr int GK = 3 * CPS / 2;              // K steps per weight granule
  constexpr int GB = GK * 2048;                // bytes per weight granule
  constexpr int PB = PKB * 1024;               // bytes per patch buffer
  constexpr int SB = 16 * CPS;                 // bytes per pixel slot
  // LDW > 0: the last LDW wavefronts only issue the LDS-direct loads and the others only multiply
  // (the loads' issue and bookkeeping instructions then stay out of the MFMA stream); LDW = 0: every
  // wavefront does both.
  constexpr int NLW = LDW ? LDW : NWV;         // wavefronts that issue loads
  constexpr int NCW = NWV - LDW;               // wavefronts that multiply
  static_assert(LDW == 0 || NC == 2, "loader wavefronts come with full-width compute wavefronts");
  constexpr int KPW = PB / 1024 / NLW;         // patch load instructions per loading wavefront per super-stage, at most
  constexpr int KH = (KPW + 1) / 2;            // of which in the first granule; the rest in the second
  constexpr int WPW = (2 * GK + NLW - 1) / NLW;   // weight load instructions per loading wavefront per granule
  // NC = 2: a wavefront multiplies its pixels by all 64 channels of the block.  NC = 1: two wavefronts
  // share a pixel fragment, one per 32-channel half (same tile on twice the wavefronts).
  static_assert(NC == 1 || NC == 2, "channel fragments per wavefront");
  constexpr int NPW = NCW * NC / 2;            // wavefronts across the pixels
  // K steps the MFMA operands are read ahead (reading three ahead measured no faster on any layer)
  constexpr int PD = 1;
  constexpr int BM = 32 * NF * NPW;            // pixels per tile
  constexpr int TAB = BM * 18 + 512 + 1024;    // bytes of tables

  // two patch buffers, the weight granule ring, tables
  __shared__ __align__(1024) char pat2[2 * PB];
  __shared__ __align__(1024) char wgt[RD * GB];
  __shared__ __align__(16) char smem[TAB];
  int* pslot = (int*)smem;                       // [BM] tile pixel -> patch slot of its tap (0,0)
  int* clist = pslot + BM;                       // [BM] compacted position -> patch slot
  uint32_t* bmp = (uint32_t*)(clist + BM);       // [BM][2] decision words of the tile
  uint16_t* rank = (uint16_t*)(bmp + 2 * BM);    // [BM] tile pixel -> compacted position
  acc_t* tlo = (acc_t*)(rank + BM);              // [64] thresholds of this channel block
  acc_t* thi = tlo + 64;
  float* aff = (float*)(thi + 64);               // [4][64] scale0, shift0, scale1, shift1 of this channel block

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  __builtin_assume(wave >= 0 && wave < NWV);
  const bool is_cw = wave < NCW;                // this wavefront multiplies
  const bool is_ld = LDW == 0 || wave >= NCW;   // this wavefront issues loads
  const int lw = LDW ? wave - NCW : wave;       // its number among the loading wavefronts
  const int pw = wave & (NPW - 1);              // which pixel fragments
  const int fc0 = NC == 2 ? 0 : wave / NPW;     // first 32-channel fragment of this wavefront
  const int lj = lane & 31, lh = lane >> 5;

  // Block id mod 8 is the XCD.  Normally the blocks that share a pixel tile (different channel blocks)
  // sit on one XCD, and an XCD takes a contiguous run of tiles, so a tile's input and the halo rows it
  // shares with its neighbours are fetched into one L2.  xcd_cb: the blocks that share a
  // channel block sit on one XCD instead, so that each L2 holds an eighth of the weights (layers whose
  // weights outweigh their input).
  int tile, cbk;
  {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    // slot / div_d without a division sequence (the launcher picks the multiplier where it is exact)
    int q;
    if (g.div_magic)
      q = (int)__umulhi((unsigned)slot, g.div_magic);
    else if (g.div_d == 1)
      q = slot;
    else
      q = slot / g.div_d;
    if (g.xcd_cb) {
      tile = q;                                     // div_d = n_cb / 8
      cbk = (slot - q * g.div_d) * 8 + xcd;
    } else {
      cbk = slot - q * g.div_d;                     // div_d = n_cb
      tile = xcd * g.tiles8 + q;                    // an XCD takes a contiguous run of tiles: neighbours share halo rows in its L2
    }
  }
  const int total_rows = p.n * p.ho;
  const int R0 = tile * g.tr;
  if (R0 >= total_rows) return;

  const int S0 = g.stages[0];                       // super-stages of the base phase
  const int S = S0 + ((p.gated && !p.gate_only) ? g.stages[1] : 0);   // a gate-only pass stops after the base phase
  const int G = 3 * S;                              // weight granules
  const int eb = g.elem_bytes;

  // weight granule j (3*super-stage + kernel row, counted over both phases) of this channel block
  // sits at wbase0 + j*GB in the base phase and at wcond0 + (j - 3*S0)*GB in the conditional phase
  const char* const wbase0 = wpk0 + (size_t)cbk * 3 * g.stages[0] * GB;
  const char* const wcond0 = wpk1 + (size_t)cbk * 3 * g.stages[1] * GB;
  // weight load instruction u of this loading wavefront: 1 KB number lw*WPW + u of the granule
  // (a loading wavefront takes WPW consecutive pieces: one address pair and immediate offsets)
  static_assert(WPW <= 3, "immediate offsets below 4 KB");
  auto issue_w = [&](const char* ws, char* dst, int u) __attribute__((always_inline)) {
    const int idx = lw * WPW + u;
    if (idx < 2 * GK) {
      const auto* gp = (const __attribute__((address_space(1))) void*)(ws + lw * (WPW * 1024) + lane * 16);
      auto* lp = (__attribute__((address_space(3))) void*)(dst + lw * (WPW * 1024));
      switch (u) {
        case 0: __builtin_amdgcn_global_load_lds(gp, lp, 16, 0, 0); break;
        case 1: __builtin_amdgcn_global_load_lds(gp, lp, 16, 1024, 0); break;
        default: __builtin_amdgcn_global_load_lds(gp, lp, 16, 2048, 0); break;
      }
    }
  };
  if (is_ld) {
#pragma unroll
    for (int u = 0; u < WPW; ++u) issue_w(wbase0, wgt, u);
  }
  const char* wnext = wbase0 + GB;   // source of the granule after the one being multiplied

  const long long m0 = (long long)R0 * p.wo;        // first output pixel
  const int rows_here = total_rows - R0 < g.tr ? total_rows - R0 : g.tr;
  const int bmv = rows_here * p.wo;                 // output pixels of this tile
  const int img0 = fdiv3(R0, g.magic_ho);
  const int rho0 = img0 * g.hp + (R0 - img0 * p.ho) * p.stride;   // stacked padded input row of patch row 0
  const int rowb = SB << g.logp;                    // bytes per patch row

  // ---- a loading wavefront's patch load instructions: instruction idx = lw + NLW*k fills the 64 chunk
  // positions [64*idx, +64), i.e. 64/CPS pixel slots; a lane outside the image keeps a zero that is
  // written once.  smask bit k: the instruction has at least one lane inside the image.
  const char* xbytes = (const char*)p.x;
  const int xps = (int)p.x_pixel_stride * eb;
  int voff[KPW];
  unsigned smask = 0u;
#pragma unroll
  for (int k = 0; k < KPW; ++k) {
    voff[k] = -1;
    const int idx = lw + NLW * k;
    if (is_ld && idx < g.ni) {
      const int pos16 = idx * 64 + lane;
      const int sl = pos16 / CPS, cp = pos16 % CPS;
      const int f = CPS == 4 ? (sl >> 2) & 3 : (sl >> 3) & 1;
      const int q = cp ^ f;
      const int prow = sl >> g.logp, c = sl & ((1 << g.logp) - 1);
      const int rho = rho0 + prow;
      const int img = fdiv3(rho, g.magic_hp);
      const int hi = rho - img * g.hp - p.pad, wi = c - p.pad;
      if (prow < g.pr && img < p.n && hi >= 0 && hi < p.h && wi >= 0 && wi < p.w) {
        voff[k] = ((img * p.h + hi) * p.w + wi) * xps + q * 16;    // the plan keeps x below 2 GiB
      } else {
        *(i32x4*)(pat2 + pos16 * 16) = i32x4{0, 0, 0, 0};
        *(i32x4*)(pat2 + PB + pos16 * 16) = i32x4{0, 0, 0, 0};
      }
      if (__ballot(voff[k] >= 0) != 0ull) smask |= 1u << k;
    }
  }
  smask = __builtin_amdgcn_readfirstlane(smask);
  // x at the first channel of super-stage sg (counted over both phases).  The base phase starts at
  // this block's first base channel; the conditional phase walks the channels in order and jumps
  // over the base channels (without grouping these are the first c_base; with grouping, Sec. 3.3,
  // those of the block's own group, or none when the block covers several groups and the packed
  // weights carry zeros instead).
  int base_ch0 = 0, gap_start = 0, gap_len = p.c_base;
  if (g.grp_mode == 1) {
    base_ch0 = gap_start = (cbk * kBn / p.cpg) * p.c_base;
  } else if (g.grp_mode == 2) {
    base_ch0 = p.groups > 1 ? cbk * g.gsp * p.c_base : 0;   // (without grouping: a base group padded with zero weights)
    gap_len = 0;
  }
  auto x_src = [&](int sg) __attribute__((always_inline)) {
    const int ph = sg >= S0 ? 1 : 0;
    const int ss = ph ? sg - S0 : sg;
    int chn = ss * CPS * g.ch;
    chn = ph ? (chn >= gap_start ? chn + gap_len : chn) : base_ch0 + chn;
    return xbytes + (long long)chn * eb;
  };
  {
    const char* xs0 = x_src(0);
#pragma unroll
    for (int k = 0; k < KPW; ++k)
      if (((smask >> k) & 1u) && voff[k] >= 0) lds_direct16(xs0 + voff[k], pat2 + (lw + NLW * k) * 1024);
  }

  // Gate thresholds of this channel block.  The loads go out after the first LDS-direct loads (an
  // ordinary load that the compiler waits for early would make it wait for those as well, before the
  // patch loads are even issued); the copy to LDS is the last thing before the first barrier.
  acc_t my_lo = 0, my_hi = 0;
  if (tid < 64) {
    const int co = cbk * kBn + tid;
    if constexpr (Base::kDtype == CG_I8) {
      my_lo = p.thr_i[co];
    } else {
      my_lo = p.thr_f[co];
      my_hi = p.thr_hi_f[co];
    }
  }

  // ---- this lane's base-path pixels ------------------------------------------------------------
  int pix[NF];
  int pimg[NF];         // image of the pixel
  bool pval[NF];
  int pa[NF][3];        // patch byte offsets of the three tap columns, kernel row 0
#pragma unroll
  for (int fp = 0; fp < NF; ++fp) {
    pix[fp] = (pw * NF + fp) * 32 + lj;
    const bool inside = pix[fp] < bmv;
    pval[fp] = is_cw && inside;
    const int i = inside ? pix[fp] : 0;             // fragments past the tile's end read pixel 0 and are dropped
    const int lr = fdiv3(i, g.magic_wo), wo_ = i - lr * p.wo;
    const int R = R0 + lr;
    const int img = fdiv3(R, g.magic_ho), hq = R - img * p.ho;
    pimg[fp] = img;
    const int slot = ((img * g.hp + hq * p.stride - rho0) << g.logp) + wo_ * p.stride;
    if (lh == 0 && is_cw) pslot[pix[fp]] = slot;
#pragma unroll
    for (int c = 0; c < 3; ++c) pa[fp][c] = slot_addr<CPS>(slot + c, lh);
  }
  for (int i = tid; i < 2 * BM; i += NT) bmp[i] = 0u;

  acc16 accP[NF][NC], accR[NF][NC];
#pragma unroll
  for (int fp = 0; fp < NF; ++fp)
#pragma unroll
    for (int fl = 0; fl < NC; ++fl)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        accP[fp][fl][i] = 0;
        accR[fp][fl][i] = 0;
      }

  unsigned dlane[NF];   // this lane's decisions of pixel fp: bit 16*fc + i = channel 32*fc + 16*lh + i
#pragma unroll
  for (int fp = 0; fp < NF; ++fp) dlane[fp] = 0u;
  int pac[NF][3];       // patch offsets of this lane's compacted pixels
#pragma unroll
  for (int fp = 0; fp < NF; ++fp)
#pragma unroll
    for (int c = 0; c < 3; ++c) pac[fp][c] = 0;
  int nrl = 0;          // compacted fragments of this wavefront
  int n_act = 0;        // fired pixels of the tile
  const int wofs = lh * 1024 + lj * 16 + fc0 * 512;   // lane's offset of its weight rows in a granule

  if (tid < 64) {
    tlo[tid] = my_lo;
    thi[tid] = my_hi;
    if (Base::kDtype != CG_I8 && (p.epilogue & CG_EPI_AFFINE)) {
      const int co = cbk * kBn + tid;
      aff[tid] = p.sc0[co];
      aff[64 + tid] = p.sh0[co];
      aff[128 + tid] = p.sc1[co];
      aff[192 + tid] = p.sh1[co];
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the first granules and the first patch have landed
  __syncthreads();

  // Per super-stage: where the next super-stage's patch comes from and which of this wavefront's
  // load instructions carry any of it (first half in the super-stage's first granule, second half in
  // its second one).
  const char* xsn = xbytes;
  bool more = false;
  int np0 = 0, np1 = 0;   // loads of this wavefront in the first / second granule (an instruction goes out iff a lane is valid)
  const int cnt0 = __popc(smask & ((1u << KH) - 1u)), cnt1 = __popc((smask >> KH) & ((1u << (KPW - KH)) - 1u));
  auto stage_setup = [&](int sg) __attribute__((always_inline)) {
    more = sg + 1 < S;
    xsn = x_src(more ? sg + 1 : sg);
    np0 = more ? cnt0 : 0;
    np1 = more ? cnt1 : 0;
  };

  // One weight granule gi (kernel row R of super-stage sg) for NL pixel fragments: multiply it out of
  // its patch buffer and ring slot; meanwhile fetch granule gi+1 into the other ring slot and, in the
  // first two granules of a super-stage, half of the next super-stage's patch into the other patch
  // buffer.  Within the granule the weight instructions go out first, then the patch instructions.
  // A wavefront's loads complete in issue order, so the closing wait for the next granule's weights
  // leaves this granule's patch loads in flight; the last granule of a super-stage waits for all.
  auto granule = [&](auto nl_tag, auto r_tag, acc16 (&acc)[NF][NC], const int (&base)[NF][3], int gi, int sg)
                     __attribute__((always_inline)) {
    constexpr int NL = decltype(nl_tag)::value;
    constexpr int R = decltype(r_tag)::value;
    constexpr int K0 = R == 1 ? KH : 0;                    // first patch instruction of this granule
    constexpr int NP = R == 0 ? KH : R == 1 ? KPW - KH : 0;   // and how many
    const char* pat = pat2 + (sg & 1) * PB;
    char* patn = pat2 + ((sg & 1) ^ 1) * PB;
    const char* wg = wgt + (gi & 1) * GB;
    char* wgn = wgt + ((gi & 1) ^ 1) * GB;
    // the kernel's very last granule has no successor: it fetches its own weights once more into the
    // free slot, which keeps the issue code free of conditions
    const char* ws = wnext;
    if (gi + 2 < G) wnext = (gi + 2 == 3 * S0) ? wcond0 : wnext + GB;
    auto part = [&](int t) __attribute__((always_inline)) {
      if constexpr (LDW > 0) {
        if (NL > 0 || !is_ld) return;      // wavefronts that multiply leave the loads to the loaders
      }
      constexpr int NU = WPW + NP;
#pragma unroll
      for (int u = (t * NU) / GK; u < ((t + 1) * NU) / GK; ++u) {
        if (u < WPW) {
          issue_w(ws, wgn, u);
        } else {
          const int i = u - WPW;
          if (more && voff[K0 + i] >= 0) lds_direct16(xsn + voff[K0 + i], patn + (lw + NLW * (K0 + i)) * 1024);
        }
      }
    };
    // the kernel row's byte offset goes through an opaque register: the three unrolled granules then
    // each form their operand addresses afresh instead of keeping all of them live across the loop
    int rofs = R * rowb;
    asm volatile("" : "+s"(rofs));
    int ar[NF][3];
#pragma unroll
    for (int fp = 0; fp < NF; ++fp)
#pragma unroll
      for (int c = 0; c < 3; ++c) ar[fp][c] = base[fp][c] + rofs;
    mma_granule<Tr, NL, NF, CPS, NC, PD>(pat, wg, wofs, ar, acc, part);
    if constexpr (LDW == 0 || NL == 0) {     // (a wavefront without loads has nothing to wait for)
      if constexpr (R == 2)
        wait_vm_upto<0>(0);
      else
        wait_vm_upto<NP>(R == 0 ? np0 : np1);
    }
  };
  // the three granules of super-stage sg
  auto super_stage = [&](auto nl_tag, acc16 (&acc)[NF][NC], const int (&base)[NF][3], int gi, int sg, bool last)
                         __attribute__((always_inline)) {
    stage_setup(sg);
    granule(nl_tag, std::integral_constant<int, 0>{}, acc, base, gi, sg);
    __builtin_amdgcn_s_barrier();
    granule(nl_tag, std::integral_constant<int, 1>{}, acc, base, gi + 1, sg);
    __builtin_amdgcn_s_barrier();
    granule(nl_tag, std::integral_constant<int, 2>{}, acc, base, gi + 2, sg);
    if (!last) __builtin_amdgcn_s_barrier();
  };

  // ---- base path --------------------------------------------------------------------------------
  int gi = 0;
#pragma nounroll
  for (int sg = 0; sg < S0; ++sg, gi += 3) {
    if (is_cw)
      super_stage(std::integral_constant<int, NF>{}, accP, pa, gi, sg, sg + 1 == S0);
    else
      super_stage(std::integral_constant<int, 0>{}, accP, pa, gi, sg, sg + 1 == S0);
  }

  if (p.gated) {
    // ---- gate -------------------------------------------------------------------------------
    uint16_t* bmph = (uint16_t*)bmp;
#pragma unroll
    for (int fp = 0; fp < NF; ++fp) {
      unsigned dl = 0u;
#pragma unroll
      for (int fl = 0; fl < NC; ++fl) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int c0 = 32 * (fc0 + fl) + 16 * lh + 4 * q4;
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
      dl <<= 16 * fc0;                 // bit 16*fc + i = channel 32*fc + 16*lh + i of the block
      if (!pval[fp]) dl = 0u;
      if (p.chan_mask) {
        // channel-wise gate (Sec. 3.2): only the channels that keep their conditional path in this image
        const uint32_t* mw = p.chan_mask + (long long)pimg[fp] * p.words + cbk * 2;
        dl &= ((mw[0] >> (16 * lh)) & 0xffffu) | (((mw[1] >> (16 * lh)) & 0xffffu) << 16);
      }
      dlane[fp] = dl;
      if (is_cw && (NC == 2 || fc0 == 0)) bmph[pix[fp] * 4 + lh] = (uint16_t)(dl & 0xffffu);
      if (is_cw && (NC == 2 || fc0 == 1)) bmph[pix[fp] * 4 + 2 + lh] = (uint16_t)(dl >> 16);
    }
    __syncthreads();

    // ---- decision words out; compaction: every wavefront scans all pixels, wavefront c places
    // pixels [64c, 64c+64)
    if (p.bitmap) {
      for (int i = tid; i < bmv; i += NT) {
        const uint2 w2 = *(const uint2*)(bmp + i * 2);
        *(uint2*)(p.bitmap + (m0 + i) * p.words + cbk * 2) = w2;
      }
    }
    if (p.gate_only) return;   // first pass of the channel-wise gate: the decisions are all it produces
    int my_prefix = 0;
    unsigned long long my_bal = 0;
#pragma unroll
    for (int c = 0; c < BM / 64; ++c) {
      const uint2 w2 = *(const uint2*)(bmp + (c * 64 + lane) * 2);
      const unsigned long long b = __ballot((w2.x | w2.y) != 0u);
      if (c == wave) {
        my_prefix = n_act;
        my_bal = b;
      }
      n_act += __popcll(b);
    }
    if ((my_bal >> lane) & 1ull) {
      const int idx = my_prefix + __popcll(my_bal & ((1ull << lane) - 1ull));
      clist[idx] = pslot[wave * 64 + lane];
      rank[wave * 64 + lane] = (uint16_t)idx;
    }
    __syncthreads();

    // compacted fragment c (32 pixels) goes to the wavefronts of pixel position c % NPW
    const int nc = (n_act + 31) >> 5;
    nrl = is_cw ? (nc > pw ? 1 : 0) + ((NF == 2 && nc > pw + NPW) ? 1 : 0) : 0;
#pragma unroll
    for (int k = 0; k < NF; ++k) {
      const int c = (pw + NPW * k) * 32 + lj;
      const int slot = clist[n_act == 0 ? 0 : (c < n_act ? c : 0)];
#pragma unroll
      for (int cc = 0; cc < 3; ++cc) pac[k][cc] = slot_addr<CPS>(slot + cc, lh);
    }

    // ---- conditional path on the listed pixels -------------------------------------------------
    if (n_act == 0) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // nothing fired: drop the phase, drain what was prefetched
      __syncthreads();
    } else {
#pragma nounroll
      for (int sg = S0; sg < S; ++sg, gi += 3) {
        if (nrl == 2) {
          if constexpr (NF == 2) super_stage(std::integral_constant<int, 2>{}, accR, pac, gi, sg, false);
        } else if (nrl == 1) {
          super_stage(std::integral_constant<int, 1>{}, accR, pac, gi, sg, false);
        } else {
          super_stage(std::integral_constant<int, 0>{}, accR, pac, gi, sg, false);
        }
      }
    }
  } else {
    __syncthreads();
  }

  // ---- combine: R (compacted rows) goes through LDS, 128 rows at a time, to the lanes that hold P ----
  if (p.gated && n_act > 0) {
    constexpr int FPP = 4;                 // compacted fragments per pass
    static_assert(FPP <= NPW && FPP * 32 * kRs <= 2 * PB, "a pass must fit the patch buffers");
    const int npass = (n_act + 32 * FPP - 1) / (32 * FPP);
    for (int q = 0; q < npass; ++q) {
      // compacted fragments FPP*q .. FPP*q+FPP-1 belong to pixel positions (FPP*q)%NPW and the
      // following ones, all in their slot (FPP*q)/NPW; a wavefront writes its channel fragments
      const int w0 = (FPP * q) & (NPW - 1), kk = (FPP * q) / NPW;
      if (pw >= w0 && pw < w0 + FPP && nrl > kk) {
        char* row = pat2 + ((pw - w0) * 32 + lj) * kRs + lh * 64;
#pragma unroll
        for (int k = 0; k < NF; ++k) {
          if (k != kk) continue;
#pragma unroll
          for (int fl = 0; fl < NC; ++fl)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              i32x4 v;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const acc_t rv = accR[k][fl][4 * q4 + e];
                v[e] = as_bits(rv);
              }
              *(i32x4*)(row + (fc0 + fl) * 128 + q4 * 16) = v;
            }
        }
      }
      __syncthreads();
#pragma unroll
      for (int fp = 0; fp < NF; ++fp) {
        if (dlane[fp]) {
          const int r = (int)rank[pix[fp]] - 32 * FPP * q;
          if (r >= 0 && r < 32 * FPP) {
            const char* row = pat2 + r * kRs + lh * 64;
#pragma unroll
            for (int fl = 0; fl < NC; ++fl)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const i32x4 v = *(const i32x4*)(row + (fc0 + fl) * 128 + q4 * 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const bool on = (dlane[fp] >> (16 * (fc0 + fl) + 4 * q4 + e)) & 1u;
                  acc_t rv;
                  from_bits(v[e], rv);
                  accP[fp][fl][4 * q4 + e] += on ? rv : (acc_t)0;
                }
              }
          }
        }
      }
      __syncthreads();
    }
  }

  // ---- output function on 16 consecutive channels per accumulator ---------------------------------
  const int ob = p.out_dtype == CG_BF16 ? 2 : p.out_dtype == CG_I8 ? 1 : 4;
  if (p.shuffle) {
    // shuffled channel order (Sec. 3.3): channel j of group i goes to position j*groups + i of its
    // pixel, one element at a time
#pragma unroll
    for (int fp = 0; fp < NF; ++fp) {
      if (!pval[fp]) continue;
#pragma unroll
      for (int fl = 0; fl < NC; ++fl) {
        const int fc = fc0 + fl;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int co = cbk * kBn + 32 * fc + 16 * lh + i;
          const int grp = co / p.cpg;
          const long long o = (m0 + pix[fp]) * p.c_out + (co - grp * p.cpg) * p.groups + grp;
          const bool fired = p.gated ? ((dlane[fp] >> (16 * fc + i)) & 1u) != 0u : true;
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
    for (int fp = 0; fp < NF; ++fp) {
      if (!pval[fp]) continue;
#pragma unroll
      for (int fl = 0; fl < NC; ++fl) {
        const int fc = fc0 + fl;
        const int co0 = cbk * kBn + 32 * fc + 16 * lh;
        const long long o = (m0 + pix[fp]) * p.c_out + co0;
        i32x4 v[4];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const acc_t sv = accP[fp][fl][4 * q4 + e];
            v[q4][e] = as_bits(sv);
          }
        const unsigned d16 = (dlane[fp] >> (16 * fc)) & 0xffffu;
        finish_store8<Base>(p, v[0], v[1], d16 & 0xffu, co0, o);
        finish_store8<Base>(p, v[2], v[3], d16 >> 8, co0 + 8, o + 8);
      }
    }
  } else {
    // 2- and 1-byte outputs: the 64 channels of a pixel form one row of an LDS tile (fragment fp of
    // every wavefront: 32*NWV rows of at most 144 bytes, inside the patch buffers), which leaves as
    // whole rows
    const int rb = kBn * ob;            // bytes per pixel row: 128 or 64
    const int rs = rb + 16;             // skewed row stride in LDS
    const bool lean = Base::kDtype != CG_I8 && p.out_dtype == CG_BF16 &&
                      !(p.epilogue & (CG_EPI_AFFINE | CG_EPI_RESIDUAL));
    const bool fastaff = Base::kDtype != CG_I8 && p.out_dtype == CG_BF16 && (p.epilogue & CG_EPI_AFFINE);
    const float relu_lo = (p.epilogue & CG_EPI_RELU) ? 0.0f : -__builtin_inff();
    static_assert(32 * NPW * 144 <= 2 * PB, "output tile must fit the patch buffers");
#pragma unroll
    for (int fp = 0; fp < NF; ++fp) {
      if (fp > 0) __syncthreads();      // the previous fragment's rows have been read
      if (is_cw) {
        char* row = pat2 + (pw * 32 + lj) * rs;
#pragma unroll
        for (int fl = 0; fl < NC; ++fl) {
          const int fc = fc0 + fl;
          const int cl = 32 * fc + 16 * lh;          // first of this lane's 16 channels in the block
          const int co0 = cbk * kBn + cl;
          const long long o = (m0 + pix[fp]) * p.c_out + co0;
          i32x4 v[4];
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const acc_t sv = accP[fp][fl][4 * q4 + e];
              v[q4][e] = as_bits(sv);
            }
          const unsigned d16 = (dlane[fp] >> (16 * fc)) & 0xffffu;
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
                const f32x4 a0 = *(const f32x4*)(aff + cl + 4 * q4), b0 = *(const f32x4*)(aff + 64 + cl + 4 * q4);
                const f32x4 a1 = *(const f32x4*)(aff + 128 + cl + 4 * q4), b1 = *(const f32x4*)(aff + 192 + cl + 4 * q4);
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
            *(i32x4*)(row + cl * 2) = o0;
            *(i32x4*)(row + cl * 2 + 16) = o2;
          } else {
            *(i32x4*)(row + cl) = i32x4{o0[0], o0[1], o2[0], o2[1]};
          }
        }
      }
      __syncthreads();
      // 16-byte pieces: piece id = row * (rb/16) + part
      const int ppr = rb >> 4;            // pieces per row: 8 or 4
      const int lpp = ppr == 8 ? 3 : 2;
      for (int id = tid; id < 32 * NPW * ppr; id += NT) {
        const int row = id >> lpp, part = id & (ppr - 1);
        const int px = ((row >> 5) * NF + fp) * 32 + (row & 31);     // tile pixel of this row
        if (px < bmv) {
          const i32x4 v = *(const i32x4*)(pat2 + row * rs + part * 16);
          *(i32x4*)((char*)p.y + ((m0 + px) * p.c_out + cbk * kBn) * ob + part * 16) = v;
        }
      }
    }
  }
}

// [c_out][9][c_phase] -> [column block][super-stage][kernel row r][K step k][chunk h][row][16 bytes]
// with tap = 3r + k / (CPS/2) and chunk = CPS*sigma + 2*(k % (CPS/2)) + h; row rho of a 32-row
// fragment holds channel 16*((rho/4)%2) + 4*(rho/8) + rho%4, which puts 16 consecutive channels in
// one lane of the transposed product
//
// Channel grouping with blocks that cover several groups (multi != 0): the base phase (phase 0)
// walks the base channels of all the block's groups, the conditional phase all c_in channels; a
// chunk that is not on that path for the row's output channel is packed as zeros (a chunk never
// straddles a group: c_base is a multiple of the chunk's channel count).
__global__ void pack_rows_kernel(const char* __restrict__ w, char* __restrict__ out, int c_phase, int eb, int ch,
                                 int cps, int stages, long long total, int multi, int phase, int c_base, int cpg) {
  const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= total) return;
  const int gk = 3 * cps / 2, pairs = cps / 2;
  const int rho = (int)(id & 63);
  long long r_ = id >> 6;
  const int h = (int)(r_ & 1);
  r_ >>= 1;
  const int k = (int)(r_ % gk);
  r_ /= gk;
  const int kr = (int)(r_ % 3);
  r_ /= 3;
  const int ss = (int)(r_ % stages);
  const int cb = (int)(r_ / stages);
  const int tap = 3 * kr + k / pairs;
  const int chunk = cps * ss + 2 * (k % pairs) + h;
  const int fc = rho >> 5, rr = rho & 31;
  const int co = cb * kBn + 32 * fc + 16 * ((rr >> 2) & 1) + 4 * (rr >> 3) + (rr & 3);
  int c_src = chunk * ch;          // first channel of the chunk in the row's w_base / w_cond
  bool zero = false;
  if (multi) {
    const int grp = co / cpg;      // the row's output group = its base input group
    if (phase == 0) {
      const int blk_grp0 = (cb * kBn) / cpg;                 // first group of this column block
      zero = blk_grp0 + c_src / c_base != grp;
      c_src = c_src % c_base;
    } else {
      zero = c_src / c_base == grp;
      if (c_src >= (grp + 1) * c_base) c_src -= c_base;
    }
  }
  i32x4 v = {0, 0, 0, 0};
  if (!zero) v = *(const i32x4*)(w + (((long long)co * 9 + tap) * c_phase + c_src) * eb);
  *(i32x4*)(out + id * 16) = v;
}

// per-(image, channel) fired counts and their total from the decision bitmap: one block per
// (image, bitmap word); a wavefront takes 64 pixels at a time and counts bit b of their words with
// a ballot, lane b keeping the running count; one atomic per block adds to the total.  With `mask`
// the block instead writes the word of the channels whose count reaches `need` (the channel-wise
// gate of Sec. 3.2) and leaves `counts` alone.
__global__ void bitmap_counts_kernel(const uint32_t* __restrict__ bitmap, int words, int hw, int c_out,
                                     uint32_t* __restrict__ counts, uint32_t* __restrict__ mask, uint32_t need) {
  __shared__ uint32_t cnt[32];
  const int w = blockIdx.x % words, img = blockIdx.x / words;
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 32) cnt[threadIdx.x] = 0u;
  __syncthreads();
  uint32_t mine = 0u;
  for (int base = (int)(threadIdx.x & ~63u); base < hw; base += (int)blockDim.x) {
    const int px = base + lane;
    const uint32_t v = px < hw ? bitmap[((long long)img * hw + px) * words + w] : 0u;
#pragma unroll
    for (int b = 0; b < 32; ++b) {
      const uint32_t nb = (uint32_t)__popcll(__ballot((v >> b) & 1u));
      mine += lane == b ? nb : 0u;
    }
  }
  if (lane < 32 && mine) atomicAdd(&cnt[lane], mine);
  __syncthreads();
  if (threadIdx.x < 64) {
    const int co = w * 32 + lane;
    uint32_t v = (lane < 32 && co < c_out) ? cnt[lane] : 0u;
    if (mask) {
      const unsigned long long keep = __ballot(lane < 32 && co < c_out && v >= need);
      if (lane == 0) mask[(long long)img * words + w] = (uint32_t)keep;
      return;
    }
    if (lane < 32 && co < c_out) counts[2 + (long long)img * c_out + co] = v;
#pragma unroll
    for (int sft = 16; sft >= 1; sft >>= 1) v += (uint32_t)__shfl_xor((int)v, sft, 64);
    if (lane == 0 && v) atomicAdd((unsigned long long*)counts, (unsigned long long)v);
  }
}

// The same for feature maps of a few pixels (fully connected layers are 1x1 maps): one thread per
// (image, bitmap word) walks the map's pixels, so a batch of thousands of tiny maps is a few hundred
// blocks and one atomic per block instead of one block and one atomic per word.
__global__ void bitmap_counts_small_kernel(const uint32_t* __restrict__ bitmap, int words, int hw, int c_out,
                                           long long items, uint32_t* __restrict__ counts,
                                           uint32_t* __restrict__ mask, uint32_t need) {
  __shared__ uint32_t part[4];
  const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t total = 0u;
  if (id < items) {
    const int w = (int)(id % words);
    const long long img = id / words;
    uint32_t keep = 0u;
    for (int b = 0; b < 32; ++b) {
      const int co = w * 32 + b;
      if (co >= c_out) break;
      uint32_t c = 0u;
      for (int px = 0; px < hw; ++px) c += (bitmap[(img * hw + px) * words + w] >> b) & 1u;
      if (mask) {
        keep |= (c >= need ? 1u : 0u) << b;
      } else {
        counts[2 + img * c_out + co] = c;
        total += c;
      }
    }
    if (mask) mask[img * words + w] = keep;
  }
  if (mask) return;
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) total += (uint32_t)__shfl_xor((int)total, sft, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = total;
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned long long v = (unsigned long long)part[0] + part[1] + part[2] + part[3];
    if (v) atomicAdd((unsigned long long*)counts, v);
  }
}

template <typename Tr, int NF, int CPS, int PKB, int NWV, int NC, int LDW>
hipError_t launch_rows_one(const Mfma3Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  const long long rows = (long long)p.n * p.ho;
  const long long tiles = (rows + g.tr - 1) / g.tr;
  const long long blocks = g.xcd_cb ? tiles * g.n_cb : ((tiles + 7) / 8) * 8 * g.n_cb;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
  if ((long long)g.ni > PKB) return hipErrorInvalidValue;     // the patch must fit its buffer (1 KB per load instruction)
  Mfma3Plan gg = g;
  gg.tiles8 = (int)((tiles + 7) / 8);
  gg.div_d = g.xcd_cb ? g.n_cb >> 3 : g.n_cb;
  gg.div_magic = 0u;
  if (gg.div_d > 1 && (blocks >> 3) * gg.div_d < (1ll << 32))   // exact for every slot of this grid
    gg.div_magic = (unsigned)(((1ull << 32) + (unsigned)gg.div_d - 1) / (unsigned)gg.div_d);
  auto kern = gated_conv_rows_kernel<Tr, NF, CPS, PKB, NWV, NC, LDW>;
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NWV * 64), 0, s, p, gg, (const char*)w0, (const char*)w1);
  return hipGetLastError();
}

template <typename Tr, int NF, int CPS>
hipError_t launch_rows_cps(const Mfma3Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (g.ldw == 4) {
    if (g.pkb == 24) return launch_rows_one<Tr, NF, CPS, 24, 8, 2, 4>(g, p, w0, w1, s);
    return launch_rows_one<Tr, NF, CPS, 48, 8, 2, 4>(g, p, w0, w1, s);
  }
  if (g.nwv == 8 && g.nc == 2) {
    if (g.pkb == 24) return launch_rows_one<Tr, NF, CPS, 24, 8, 2, 0>(g, p, w0, w1, s);
    return launch_rows_one<Tr, NF, CPS, 48, 8, 2, 0>(g, p, w0, w1, s);
  }
  if (g.nwv == 8) {
    if (g.pkb == 24) return launch_rows_one<Tr, NF, CPS, 24, 8, 1, 0>(g, p, w0, w1, s);
    return launch_rows_one<Tr, NF, CPS, 48, 8, 1, 0>(g, p, w0, w1, s);
  }
  if (g.pkb == 24) return launch_rows_one<Tr, NF, CPS, 24, 4, 2, 0>(g, p, w0, w1, s);
  return launch_rows_one<Tr, NF, CPS, 48, 4, 2, 0>(g, p, w0, w1, s);
}

template <typename Tr>
hipError_t launch_rows_dtype(const Mfma3Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (g.nf != 1) return hipErrorInvalidValue;   // the plan only issues one fragment per wavefront
  if (g.cps == 4) return launch_rows_cps<Tr, 1, 4>(g, p, w0, w1, s);
  return launch_rows_cps<Tr, 1, 2>(g, p, w0, w1, s);
}

unsigned magic_of3(int d) { return d == 1 ? 0u : (unsigned)(((1ull << 32) + (unsigned)d - 1) / (unsigned)d); }

}  // namespace

namespace {
Mfma3Plan plan_with(const cg_conv_desc& d, int max_cps, int n_cu, bool strict);
}

Mfma3Plan mfma3_plan(const cg_conv_desc& d, int n_cu) {
  Mfma3Plan g = plan_with(d, 4, n_cu, true);
  if (g.ok && g.cps == 4 && g.pkb == 48) {
    // Four-chunk super-stages need the 48 KB patch buffers here (one workgroup per CU).  If the grid has
    // more workgroups than CUs and two-chunk super-stages fit the 24 KB class, two workgroups per CU
    // with twice the granules are faster (stride-2 layers: 128->256 at 28x28 -20 %).
    const int ho = (d.h + 2 * d.pad - 3) / d.stride + 1;
    const long long wg = (((long long)d.n_max * ho + g.tr - 1) / g.tr) * g.n_cb;
    if (wg > n_cu) {
      const Mfma3Plan h = plan_with(d, 2, n_cu, true);
      if (h.ok && h.pkb == 24) return h;
    }
  }
  // Wide images with a large patch per output row (stride 2, many channels per super-stage): two-chunk
  // super-stages halve the patch; failing that, a tile that fills less than three quarters of its
  // pixel slots still beats the plain kernel by far.
  if (!g.ok) g = plan_with(d, 2, n_cu, true);
  if (!g.ok) g = plan_with(d, 4, n_cu, false);
  if (!g.ok) g = plan_with(d, 2, n_cu, false);
  return g;
}

namespace {
Mfma3Plan plan_with(const cg_conv_desc& d, int max_cps, int n_cu, bool strict) {
  Mfma3Plan g{};
  g.ok = 0;
  if (d.in_dtype != CG_BF16 && d.in_dtype != CG_I8) return g;
  if (d.kh != 3 || d.kw != 3) return g;
  if (d.stride < 1 || d.stride > 2 || d.pad > 1) return g;
  g.elem_bytes = d.in_dtype == CG_BF16 ? 2 : 1;
  g.ch = 16 / g.elem_bytes;
  const long long xps = d.x_pixel_stride ? d.x_pixel_stride : d.c_in;
  if (xps % g.ch) return g;
  // channels the two phases walk
  int base_k = d.c_base, c_cond = d.c_in - d.c_base;
  g.grp_mode = 0;
  g.gsp = 1;
  if (d.groups > 1) {
    const int cpg = d.c_out / d.groups;
    if (cpg % kBn == 0) {
      g.grp_mode = 1;                       // a 64-channel block lies inside one group
    } else if (kBn % cpg == 0 && d.c_base % g.ch == 0) {
      g.grp_mode = 2;                       // a block covers kBn/cpg whole groups
      g.gsp = kBn / cpg;
      base_k = g.gsp * d.c_base;
      c_cond = d.c_in;
    } else {
      return g;
    }
  }
  if (d.groups <= 1 && base_k % (2 * g.ch) != 0 && base_k % g.ch == 0 && base_k < d.c_in &&
      d.c_in % (2 * g.ch) == 0) {
    // A base group of one 16-byte chunk (16 int8 channels) is below the two-chunk K granule: the base
    // phase then walks two chunks with zero weights on the second, and the conditional phase all
    // input channels with zero weights on the base ones - the packing of a block that covers
    // several groups, with one group.
    g.grp_mode = 2;
    g.gsp = 2;
    base_k = 2 * d.c_base;
    c_cond = d.c_in;
  }
  if (max_cps >= 4 && base_k % (4 * g.ch) == 0 && c_cond % (4 * g.ch) == 0)
    g.cps = 4;
  else if (base_k % (2 * g.ch) == 0 && c_cond % (2 * g.ch) == 0)
    g.cps = 2;
  else
    return g;
  if (d.c_out % kBn) return g;
  const int ho = (d.h + 2 * d.pad - 3) / d.stride + 1, wo = (d.w + 2 * d.pad - 3) / d.stride + 1;
  // 32-bit byte offsets and 16-bit row numbers inside the kernel
  if ((long long)d.n_max * d.h * d.w * xps * g.elem_bytes >= (1ll << 31)) return g;
  if ((long long)d.n_max * ho * wo >= (1ll << 30)) return g;
  if ((long long)d.n_max * (d.h + 2 * d.pad) >= 65536 || (long long)d.n_max * ho >= 65536) return g;
  g.n_cb = d.c_out / kBn;
  g.hp = d.h + 2 * d.pad;
  g.magic_hp = magic_of3(g.hp);
  g.magic_ho = magic_of3(ho);
  g.magic_wo = magic_of3(wo);
  g.logp = 4;
  while ((1 << g.logp) < d.w + d.pad) ++g.logp;
  if ((1 << g.logp) == d.w + d.pad && d.pad) ++g.logp;   // keep a zero slot after the last column
  if (g.logp > 8) return g;
  const int P = 1 << g.logp;
  const int sb = 16 * g.cps;
  const long long rows = (long long)d.n_max * ho;
  auto gcd = [](int a, int b) {
    while (b) {
      const int t = a % b;
      a = b;
      b = t;
    }
    return a;
  };
  // patch rows of a tile of t output rows, maximum over the tile starts that occur (multiples of t)
  auto patch_rows = [&](int t) {
    int pr = 0;
    const int step = gcd(t, ho);
    for (int r0 = 0; r0 < ho; r0 += step) {
      const int r1 = r0 + t - 1;
      const int rows_here = (r1 / ho) * g.hp + (r1 % ho) * d.stride - r0 * d.stride + 3;
      if (rows_here > pr) pr = rows_here;
    }
    return pr;
  };
  // Candidates in order of preference: 24 KB patch buffers (two workgroups per CU), then 48 KB.
  // Within a class the large tile comes first; a candidate must keep three quarters of its pixel
  // slots busy.  (Eight-wavefront workgroups, one per CU with the weights fetched three granules
  // ahead, measured slower than two four-wavefront workgroups on every benchmark layer; the kernel
  // template still takes the wavefront count.)
  struct Cand {
    int nwv, pkb;
    long long min_wg;
  };
  const Cand cands[] = {{4, 24, 0}, {4, 48, 0}};
  for (const Cand& c : cands) {
    for (int nf = 2; nf >= 1; --nf) {
      const int bm = 32 * nf * c.nwv;
      int tr = bm / wo;
      if (tr < 1) continue;
      if (tr > rows) tr = (int)rows;
      int t = tr;
      while (t >= 1 && (long long)patch_rows(t) * P * sb > c.pkb * 1024) --t;
      if (t < 1 || (strict && 4 * t < 3 * tr)) continue;
      if (nf == 2 && ((rows + t - 1) / t) * g.n_cb < n_cu) continue;   // the large tile only when it still fills the CUs
      {
        // Balance the grid: with fewer rows per tile the tiles may come out as a whole number of
        // rounds over the CUs (two workgroups each where LDS allows), which shortens the
        // longest CU's share.  Cost of a choice = rounds x (rows per tile + a per-round share for
        // prologue, gate and epilogue); ties keep the larger tile.
        const int gkb = 3 * g.cps;
        const long long slots = (long long)n_cu * ((2 * c.pkb + 2 * gkb + 6 <= 80) ? 2 : 1);
        const int tmax = t;
        double best = 1e30;
        // (with more than two rounds the workgroups no longer run in step and the larger tile wins)
        if ((((rows + tmax - 1) / tmax) * g.n_cb + slots - 1) / slots <= 2)
        for (int tt = tmax; 4 * tt >= 3 * tr && tt >= 1; --tt) {     // (three quarters of the pixel slots stay in use)
          // (a shorter tile may straddle images where the longer one does not, and then needs more patch rows)
          if ((long long)patch_rows(tt) * P * sb > c.pkb * 1024) continue;
          const long long wg = ((rows + tt - 1) / tt) * g.n_cb;
          const long long rounds = (wg + slots - 1) / slots;
          const double cost = (double)rounds * (tt + 0.35 * tmax);
          if (cost < best - 1e-9) {
            best = cost;
            t = tt;
          }
        }
      }
      const long long tiles = (rows + t - 1) / t;
      if (tiles * g.n_cb < c.min_wg) continue;
      g.nwv = c.nwv;
      g.nf = nf;
      g.nc = 2;
      g.ldw = 0;
      if (nf == 1 && c.pkb == 24 && tiles * g.n_cb <= n_cu) {
        // a small tile that is alone on its CU because the grid has no second one to offer: four
        // more wavefronts take over the LDS-direct loads (measured 5-8 % faster on the 512-channel
        // 7x7 layer; slower where two workgroups share a CU)
        g.nwv = 8;
        g.ldw = 4;
      }
      if (nf == 1 && c.pkb == 48 && g.ldw == 0) {
        // a tile that is alone on its CU (large patch buffers): eight wavefronts, two per pixel
        // fragment with 32 channels each, measured 5-10 % faster there than four with 64
        g.nwv = 8;
        g.nc = 1;
      }
      if (nf == 2) {
        // the 256-pixel tile runs as eight wavefronts of one fragment each rather than four of two:
        // same tile, half the registers per wavefront, twice the wavefronts to overlap each other's
        // scalar work and waits (measured 8-10 % faster on the 64- and 128-channel layers)
        g.nwv = 8;
        g.nf = 1;
      }
      // which operand an XCD's L2 should see whole: the heavier one (512-channel 7x7 layer: -11 %)
      g.xcd_cb = (g.n_cb % 8 == 0 && 9ll * d.c_in * d.c_out > (long long)d.n_max * d.h * d.w * d.c_in) ? 1 : 0;
      g.bm = bm;
      g.tr = t;
      g.pkb = c.pkb;
      g.pr = patch_rows(t);
      g.ni = (g.pr * P * g.cps + 63) / 64;
      g.stages[0] = base_k / (g.cps * g.ch);
      g.stages[1] = c_cond / (g.cps * g.ch);
      const size_t gb = (size_t)(3 * g.cps / 2) * 2048;
      g.wpk_base_bytes = (size_t)g.n_cb * g.stages[0] * 3 * gb;
      g.wpk_cond_bytes = (size_t)g.n_cb * g.stages[1] * 3 * gb;
      g.ok = 1;
      return g;
    }
  }
  return g;
}
}  // namespace

hipError_t launch_mfma3_pack(const Mfma3Plan& g, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s) {
  for (int ph = 0; ph < 2; ++ph) {
    if (g.stages[ph] == 0) continue;
    const long long total = (long long)g.n_cb * g.stages[ph] * 3 * (3 * g.cps / 2) * 2 * 64;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_rows_kernel, dim3(blocks), dim3(256), 0, s, (const char*)(ph ? p.w_cond : p.w_base),
                       (char*)(ph ? wpk_cond : wpk_base), ph ? p.c_cond : p.c_base, g.elem_bytes, g.ch, g.cps,
                       g.stages[ph], total, g.grp_mode == 2 ? 1 : 0, ph, p.c_base, p.cpg);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_mfma3(const Mfma3Plan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  if (p.in_dtype == CG_BF16) return launch_rows_dtype<Bf16Rows>(g, p, w0, w1, s);
  return launch_rows_dtype<I8Rows>(g, p, w0, w1, s);
}

namespace {
constexpr int kSmallMap = 16;   // pixels per feature map up to which the per-thread counting kernel is used
}

hipError_t launch_bitmap_counts(const Params& p, const uint32_t* bitmap, hipStream_t s) {
  const long long blocks = (long long)p.n * p.words;
  if (blocks <= 0) return hipSuccess;
  if (p.ho * p.wo <= kSmallMap) {
    hipLaunchKernelGGL(bitmap_counts_small_kernel, dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, s, bitmap,
                       p.words, p.ho * p.wo, p.c_out, blocks, p.counts, (uint32_t*)nullptr, 0u);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(bitmap_counts_kernel, dim3((unsigned)blocks), dim3(256), 0, s, bitmap, p.words, p.ho * p.wo,
                     p.c_out, p.counts, (uint32_t*)nullptr, 0u);
  return hipGetLastError();
}

hipError_t launch_bitmap_chan_mask(const Params& p, const uint32_t* bitmap, uint32_t need, uint32_t* mask,
                                   hipStream_t s) {
  const long long blocks = (long long)p.n * p.words;
  if (blocks <= 0) return hipSuccess;
  if (p.ho * p.wo <= kSmallMap) {
    hipLaunchKernelGGL(bitmap_counts_small_kernel, dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, s, bitmap,
                       p.words, p.ho * p.wo, p.c_out, blocks, (uint32_t*)nullptr, mask, need);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(bitmap_counts_kernel, dim3((unsigned)blocks), dim3(256), 0, s, bitmap, p.words, p.ho * p.wo,
                     p.c_out, (uint32_t*)nullptr, mask, need);
  return hipGetLastError();
}

}  // namespace cg
