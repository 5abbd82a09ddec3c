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

  // call arguments
  const void* x;
  const void* residual;
  void* y;
  uint32_t* bitmap;
  uint32_t* counts;
};

// Geometry of the matrix-core kernels for one layer (host-computed, passed by value).
//
// A workgroup owns a tile of up to 128 output pixels (`ti` whole images or `tr` output
// rows of one image) times BN output channels.  The input patch those pixels read is
// staged in LDS once per K stage, `cbq` 16-byte channel chunks per pixel at a time,
// together with the matching slice of prepacked weights.  Phase 0 is the base path
// (channels [0,c_base)), phase 1 the conditional path.
struct MfmaPlan {
  int ok;                  // 0: shape not covered by the matrix-core kernels
  int elem_bytes;          // 2 (bf16) or 1 (int8)
  int ch;                  // channels per 16-byte chunk: 8 (bf16) or 16 (int8)
  int bn;                  // output channels per workgroup (64 or 128)
  int n_cb;                // c_out / bn
  int tr, ti;              // output rows per tile / images per tile (ti > 1 only with tr == ho)
  int tiles_per_img;       // ceil(ho / tr) when ti == 1
  int pr, pwid, npix;      // patch rows, patch width, patch pixels = ti*pr*pwid
  int bm_valid;            // ti*tr*wo output pixels per full tile (<= 128)
  int ng;                  // 16-pixel row groups per tile = ceil(bm_valid / 16)
  int taps;                // kh*kw
  int cbq[2];              // 16-byte chunks per pixel per stage
  int stages[2];           // K stages per phase (0 for an absent phase)
  int tsteps[2];           // MFMA K steps per stage = ceil(taps*cbq / 4)
  int ps[2];               // LDS bytes per patch pixel (odd multiple of 16: conflict-free reads)
  // LDS byte offsets
  int lds_aoff, lds_gidx, lds_outpp, lds_outm, lds_colcnt, lds_dbits, lds_stage, lds_w[2], lds_total;
  size_t wpk_stage_bytes[2];  // bytes of one (column block, stage) slice of prepacked weights
  size_t wpk_base_bytes, wpk_cond_bytes;
};

MfmaPlan mfma_plan(const cg_conv_desc& d);

// Geometry of the pixel-compacting matrix-core kernel.
//
// Output rows of the whole batch are numbered R = img*Ho + ho.  A workgroup owns `tr`
// consecutive global rows (<= bm pixels, they may straddle images) x 64 output channels.
// Input rows live in a "stacked padded" space, row = img*(H+2*pad) + hi + pad, in which the
// rows a tile reads form one contiguous range even across an image boundary.
struct Mfma2Plan {
  int ok;
  int elem_bytes, ch;      // bytes per element; channels per 16-byte chunk
  int ngw;                 // 16-pixel row groups per wavefront in the base phase (1 or 2)
  int bm;                  // ngw*16*wavefronts: pixels per tile, padded
  int n_cb;                // c_out / 64
  int tr;                  // global output rows per tile
  int hp;                  // h + 2*pad
  unsigned magic_hp, magic_ho, magic_wo;   // ceil(2^32 / d): exact division of 16-bit values by hp, ho, wo
  int pr_max, pw, npix;    // patch rows (max over tiles), patch width, pr_max*pw
  int bm_valid;            // tr*wo
  int ng;                  // ceil(bm_valid/16)
  int max_imgs;            // images one tile can touch
  int cbq;                 // 16-byte channel chunks per pixel per K stage: 1, 2 or 4
  int stages[2];           // K stages of the base / conditional phase
  int tsteps;              // MFMA K steps per stage = ceil(9*cbq/4)
  int kp;                  // patch chunk slots per thread per stage
  int pln, nps;            // bytes / 16-byte slots per chunk plane of the LDS patch (npix pixels + a zero pixel, padded)
  unsigned magic_nps;
  int patch_bytes, w_bytes, stage_bytes;
  int lds_goff, lds_outpp, lds_outm, lds_flag, lds_clist, lds_rank, lds_dbits, lds_colcnt, lds_zero, lds_misc,
      lds_stage, lds_total;
  size_t wpk_stage_bytes, wpk_base_bytes, wpk_cond_bytes;
};

Mfma2Plan mfma2_plan(const cg_conv_desc& d);
hipError_t launch_mfma2_pack(const Mfma2Plan& plan, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s);
hipError_t launch_mfma2(const Mfma2Plan& plan, const Params& p, const void* wpk_base, const void* wpk_cond,
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
  int stages[2];           // super-stages of the base / conditional phase
  size_t wpk_base_bytes, wpk_cond_bytes;
};

Mfma3Plan mfma3_plan(const cg_conv_desc& d);
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
hipError_t launch_mfma_pack(const MfmaPlan& plan, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s);
hipError_t launch_mfma(const MfmaPlan& plan, const Params& p, const void* wpk_base, const void* wpk_cond,
                       hipStream_t s);

}  // namespace cg
