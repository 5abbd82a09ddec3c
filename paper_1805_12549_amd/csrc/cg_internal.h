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
  int groups;              // >= 1; > 1: channel grouping (Sec. 3.3), output group i has input group i as base
  int cpg;                 // output channels per group = c_out / groups
  int shuffle;             // y (and the residual) in shuffled channel order: channel j of group i at j*groups + i
  int gate_only;           // first pass of the channel-wise gate: base path and gate only; writes the bitmap
                           // (row-tiled kernel) or the per-(image, channel) counts (plain kernel), nothing else
  const uint32_t* chan_mask;  // second pass: [n][words] bits of the channels that keep their conditional
                              // path (Sec. 3.2 channel-wise gate), ANDed into the decisions; or NULL

  // per-output-channel tables, device, in `packed`
  const float* thr_f;      // lower threshold on the fp32 base sum (Sec. 3.2 merged gate)
  const float* thr_hi_f;   // upper threshold (+inf when one-sided)
  const int32_t* thr_i;    // integer threshold (int8 path)
  const float *sc0, *sh0, *sc1, *sh1;
  const int32_t *mult0, *mult1, *bias;

  // weights in caller layout [c_out][kh][kw][c], copied into `packed`
  const void* w_base;
  const void* w_cond;
  size_t table_stride;     // bytes between the per-channel tables of `packed`; thr_f is table 0
  const void* zeros;       // at least 256 bytes of zeros (source of the padding in the LDS-direct loads)

  // call arguments
  const void* x;
  const void* residual;
  void* y;
  uint32_t* bitmap;
  uint32_t* counts;
};

// Geometry of the large-tile matrix-core kernel (kernels_tile.hip): four wavefronts per workgroup,
// one workgroup per compute unit, a wavefront multiplies `fp` 32-pixel fragments by 64 channels.
// K is walked in stages of `cps` 16-byte channel chunks per pixel times all taps.
struct TilePlan {
  int ok;
  int elem_bytes, ch;      // bytes per element; channels per 16-byte chunk
  int taps;                // 9 (3x3) or 1 (1x1)
  int cps;                 // chunks per pixel per stage
  int fp;                  // 32-pixel fragments per wavefront: 4, 2 or 1
  int wn;                  // wavefronts across the channels: 1 (64-channel block) or 2 (128)
  int bn, n_cb;            // channels per block, number of blocks
  int flat, vw;            // flat: a 1x1 stride-1 layer walked as one image of rows of vw pixels
  int tr;                  // output rows per tile
  int hp;                  // h + 2*pad of the geometry walked (for n_max)
  int logp;                // log2 of the patch row pitch in pixel slots
  int pr;                  // patch rows, maximum over tiles
  int n16;                 // 16-byte positions of a stage's patch = pr * pitch * cps
  int xcd_cb;              // 1: blocks of one channel block share an XCD; 0: blocks of one tile do
  int grp_mode, gsp;       // channel grouping, as in Mfma3Plan
  int stages[2];           // stages of the base / conditional phase
  int nb;                  // stage buffers in LDS (the loads run nb - 1 stages ahead)
  size_t lds_bytes;        // LDS of the kernel instantiation
  size_t wpk_stage_bytes;  // bytes of one (channel block, stage) slab of prepacked weights
  size_t wpk_base_bytes, wpk_cond_bytes;
};

// the image geometry the kernel walks for one call (the layer's own, or the flat renumbering)
struct TileGeo {
  int n, h, w, ho, wo, stride, pad, hp;
  unsigned magic_hp, magic_ho, magic_wo;
  long long m_valid;       // output pixels
  long long in_valid;      // input pixels
  int xps;                 // bytes between input pixels
};

TilePlan tile_plan(const cg_conv_desc& d, int n_cu);
hipError_t launch_tile_pack(const TilePlan& plan, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s);
hipError_t launch_tile(const TilePlan& plan, const Params& p, const void* wpk_base, const void* wpk_cond,
                       hipStream_t s);
// one translation unit per (dtype, kernel size): the instantiations of the tile kernel
hipError_t launch_tile_bf16_k3(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                               hipStream_t s);
hipError_t launch_tile_bf16_k1(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                               hipStream_t s);
hipError_t launch_tile_i8_k3(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                             hipStream_t s);
hipError_t launch_tile_i8_k1(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                             hipStream_t s);

// Geometry of the row-tiled matrix-core kernel (32x32 MFMA blocks, transposed product).
//
// Tiles are `tr` consecutive global output rows x 64 channels as above.  K is walked in super-stages
// of `cps` 16-byte channel chunks per pixel; the LDS patch of a super-stage holds 16*cps bytes per
// pixel slot, slot = patch_row * 2^logp + (wi + pad).
struct Mfma3Plan {
  int ok;
  int elem_bytes, ch;      // bytes per element; channels per 16-byte chunk
  int nwv;                 // wavefronts per workgroup: 4, or 8 for the 256-pixel tile
  int nf;                  // 32-pixel fragments per wavefront in the base phase
  int nc;                  // 32-channel fragments per wavefront: 2, or 1 when two wavefronts share a pixel fragment
  int ldw;                 // wavefronts (of nwv) that only issue the LDS-direct loads: 0 or 4
  int xcd_cb;              // 1: blocks of one channel block share an XCD (needs n_cb % 8 == 0); 0: blocks of one tile do
  int bm;                  // 32*nf*nwv*nc/2 pixels per tile, padded
  int n_cb;                // c_out / 64
  int tr;                  // global output rows per tile
  int hp;                  // h + 2*pad
  unsigned magic_hp, magic_ho, magic_wo;
  int logp;                // log2 of the patch row pitch in pixel slots (pitch >= 16, > w + pad - 1)
  int pr;                  // patch rows, maximum over tiles
  int cps;                 // chunks per pixel per super-stage: 4 or 2
  int ni;                  // 1 KB load instructions per super-stage patch = ceil(pr * pitch * cps / 64)
  int pkb;                 // LDS patch buffer class: 24 KB (two workgroups per CU) or 48 KB
  // Channel grouping.  0: none.  1: a 64-channel block lies inside one output group; its base
  // channels start at group*c_base and the conditional phase skips them.  2: a block covers
  // `gsp` whole groups; its base phase walks the gsp*c_base base channels of all of them and its
  // conditional phase all c_in channels, the packed weights holding zeros where a channel is not on
  // that path for that output channel.
  int grp_mode, gsp;
  // set by the launcher for the call's grid: ceil(tiles / 8); the divisor that splits a block slot into
  // (tile, channel block) and its multiplier (0: divide)
  int tiles8, div_d;
  unsigned div_magic;
  int stages[2];           // super-stages of the base / conditional phase
  size_t wpk_base_bytes, wpk_cond_bytes;
};

Mfma3Plan mfma3_plan(const cg_conv_desc& d, int n_cu);
hipError_t launch_mfma3_pack(const Mfma3Plan& plan, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s);
hipError_t launch_mfma3(const Mfma3Plan& plan, const Params& p, const void* wpk_base, const void* wpk_cond,
                        hipStream_t s);
// per-(image, channel) fired counts and their total (into p.counts, total pre-zeroed) from a decision bitmap
hipError_t launch_bitmap_counts(const Params& p, const uint32_t* bitmap, hipStream_t s);
// channel-wise gate: mask[img][w] bit b = (fired count of channel 32*w + b in image img, from the bitmap) >= need
hipError_t launch_bitmap_chan_mask(const Params& p, const uint32_t* bitmap, uint32_t need, uint32_t* mask,
                                   hipStream_t s);

// channel-wise gate: mask[img][w] bit b = counts[2 + img*c_out + 32*w + b] >= need
hipError_t launch_chan_mask(const uint32_t* counts, int n, int c_out, int words, uint32_t need, uint32_t* mask,
                            hipStream_t s);

// launchers (return hipError_t from the last launch)
hipError_t launch_naive(const Params& p, hipStream_t s);
hipError_t launch_zero_u32(uint32_t* ptr, size_t words, hipStream_t s);

}  // namespace cg
