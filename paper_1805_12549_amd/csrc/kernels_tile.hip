// Host side of the large-tile matrix-core kernel (tile_kernel.h): the plan that picks a tile
// shape for a layer, the weight prepack and the launch geometry.
#include <cstdlib>

#include "cg_mfma_common.h"
#include "tile_cfg.h"

namespace cg {

namespace {

// [c_out][taps][c_phase] -> [column block][stage][K step k][lane half h][row][16 bytes], each stage
// padded to a multiple of 4 KB.  Unit u = 2k + h of a stage is (tap u / cps, chunk cps*stage + u % cps);
// units past the last tap are zeros.  Row rho of a 32-row fragment holds channel
// 16*((rho/4)%2) + 4*(rho/8) + rho%4, which puts 16 consecutive channels in one lane of the
// transposed product.
//
// Channel grouping with blocks that cover several groups (multi != 0): the base phase (phase 0)
// walks the base channels of all the block's groups, the conditional phase all c_in channels; a
// chunk that is not on that path for the row's output channel is packed as zeros (a chunk never
// straddles a group: c_base is a multiple of the chunk's channel count).
__global__ void pack_tile_kernel(const char* __restrict__ w, char* __restrict__ out, int c_phase, int eb, int ch,
                                 int cps, int taps, int bn, int ks, int stage_bytes, int stages, long long total,
                                 int multi, int phase, int c_base, int cpg) {
  const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= total) return;
  const int per_stage = stage_bytes / 16;
  const int in_stage = (int)(id % per_stage);
  const long long st = id / per_stage;
  const int ss = (int)(st % stages);
  const int cb = (int)(st / stages);
  i32x4 v = {0, 0, 0, 0};
  const int rho = in_stage % bn;
  const int hk = in_stage / bn;
  const int h = hk & 1, k = hk >> 1;
  const int u = 2 * k + h;
  const int tap = u / cps;
  if (k < ks && tap < taps) {
    const int chunk = cps * ss + u % cps;
    const int fc = rho >> 5, rr = rho & 31;
    const int co = cb * bn + 32 * fc + 16 * ((rr >> 2) & 1) + 4 * (rr >> 3) + (rr & 3);
    int c_src = chunk * ch;          // first channel of the chunk in the row's w_base / w_cond
    bool zero = false;
    if (multi) {
      const int grp = co / cpg;      // the row's output group = its base input group
      if (phase == 0) {
        const int blk_grp0 = (cb * bn) / cpg;                  // first group of this column block
        zero = blk_grp0 + c_src / c_base != grp;
        c_src = c_src % c_base;
      } else {
        zero = c_src / c_base == grp;
        if (c_src >= (grp + 1) * c_base) c_src -= c_base;
      }
    }
    if (!zero) v = *(const i32x4*)(w + (((long long)co * taps + tap) * c_phase + c_src) * eb);
  }
  *(i32x4*)(out + id * 16) = v;
}

unsigned magic_of(int d) { return d == 1 ? 0u : (unsigned)(((1ull << 32) + (unsigned)d - 1) / (unsigned)d); }

// the geometry the kernel walks for a call of n images
TileGeo make_geo(const TilePlan& g, const Params& p) {
  TileGeo q{};
  const long long m = (long long)p.n * p.ho * p.wo;
  if (g.flat) {
    q.n = 1;
    q.w = q.wo = g.vw;
    q.h = q.ho = (int)((m + g.vw - 1) / g.vw);
    q.stride = 1;
    q.pad = 0;
  } else {
    q.n = p.n;
    q.h = p.h;
    q.w = p.w;
    q.ho = p.ho;
    q.wo = p.wo;
    q.stride = p.stride;
    q.pad = p.pad;
  }
  q.hp = q.h + 2 * q.pad;
  q.magic_hp = magic_of(q.hp);
  q.magic_ho = magic_of(q.ho);
  q.magic_wo = magic_of(q.wo);
  q.m_valid = m;
  q.in_valid = (long long)p.n * p.h * p.w;
  q.xps = (int)(p.x_pixel_stride * g.elem_bytes);
  return q;
}

}  // namespace

namespace {
// the (taps, cps, fp, wn) combinations the instantiation units provide
bool has_kernel(int taps, int cps, int fp, int wn) {
  if (taps == 9) {
    if (cps == 2) return true;
    if (cps == 4) return wn == 1 && fp <= 2;
    if (cps == 1) return wn == 1;
    return false;
  }
  if (cps == 8 || cps == 4) return true;
  if (cps == 2) return fp <= 2;
  return false;
}

TilePlan plan_wn(const cg_conv_desc& d, int n_cu, int wn) {
  const int hint_fp = d.tile_hint & 15, hint_cps = (d.tile_hint >> 8) & 15;
  TilePlan g{};
  g.ok = 0;
  if (d.in_dtype != CG_BF16 && d.in_dtype != CG_I8) return g;
  const bool k3 = d.kh == 3 && d.kw == 3, k1 = d.kh == 1 && d.kw == 1;
  if (!k3 && !k1) return g;
  if (d.stride < 1 || d.stride > 2 || d.pad < 0 || d.pad > (k3 ? 1 : 0)) return g;
  g.taps = k3 ? 9 : 1;
  g.elem_bytes = d.in_dtype == CG_BF16 ? 2 : 1;
  g.ch = 16 / g.elem_bytes;
  const long long xps = d.x_pixel_stride ? d.x_pixel_stride : d.c_in;
  if (xps % g.ch) return g;
  if (d.c_out % 64) return g;
  // channels the two phases walk
  int base_k = d.c_base, c_cond = d.c_in - d.c_base;
  g.grp_mode = 0;
  g.gsp = 1;
  if (d.c_out % (64 * wn)) return g;
  if (d.groups > 1) {
    const int cpg = d.c_out / d.groups;
    const int bn = 64 * wn;
    if (cpg % bn == 0) {
      g.grp_mode = 1;                       // a channel block lies inside one group
    } else if (bn % cpg == 0 && d.c_base % g.ch == 0) {
      g.grp_mode = 2;                       // a block covers bn/cpg whole groups
      g.gsp = bn / cpg;
      base_k = g.gsp * d.c_base;
      c_cond = d.c_in;
    } else {
      return g;
    }
  }
  if (base_k % g.ch || c_cond % g.ch) return g;
  const int bchunks = base_k / g.ch, cchunks = c_cond / g.ch;
  auto divides = [&](int c) { return bchunks % c == 0 && cchunks % c == 0; };
  if (k3) {
    const int want = hint_cps ? hint_cps : 2;
    g.cps = (want >= 4 && divides(4)) ? 4 : (want >= 2 && divides(2)) ? 2 : 1;
  } else {
    g.cps = divides(8) ? 8 : divides(4) ? 4 : divides(2) ? 2 : 0;
    if (!g.cps) return g;
  }
  g.wn = wn;
  g.bn = 64 * wn;
  g.n_cb = d.c_out / g.bn;
  const int ho = (d.h + 2 * d.pad - d.kh) / d.stride + 1, wo = (d.w + 2 * d.pad - d.kw) / d.stride + 1;
  const long long m_max = (long long)d.n_max * ho * wo;
  // 32-bit byte offsets and 16-bit row numbers inside the kernel
  if ((long long)d.n_max * d.h * d.w * xps * g.elem_bytes >= (1ll << 31)) return g;
  if (m_max >= (1ll << 30)) return g;
  g.flat = (k1 && d.stride == 1 && d.pad == 0) ? 1 : 0;
  int vh = d.h, vw = d.w, vho = ho, vwo = wo, vstride = d.stride, vpad = d.pad;
  long long rows = (long long)d.n_max * ho;
  if (g.flat) {
    vw = 64;
    while (vw < 256 && (m_max + vw - 1) / vw >= 65536) vw *= 2;
    g.vw = vw;
    vwo = vw;
    rows = (m_max + vw - 1) / vw;
    vh = vho = (int)rows;
    vstride = 1;
    vpad = 0;
    if (rows >= 65536) return g;
  } else {
    if ((long long)d.n_max * (d.h + 2 * d.pad) >= 65536 || rows >= 65536) return g;
  }
  const int hp = vh + 2 * vpad;
  g.logp = 4;
  while ((1 << g.logp) < vw + vpad) ++g.logp;
  if ((1 << g.logp) == vw + vpad && vpad) ++g.logp;   // keep a zero slot after the last column
  if (g.logp > 8) return g;
  const int P = 1 << g.logp;
  auto gcd = [](int a, int b) {
    while (b) {
      const int t = a % b;
      a = b;
      b = t;
    }
    return a;
  };
  // patch rows of a tile of t output rows, maximum over the tile starts that occur (multiples of t)
  const int kh = d.kh;
  auto patch_rows = [&](int t) {
    int pr = 0;
    const int step = gcd(t, vho);
    for (int r0 = 0; r0 < vho; r0 += step) {
      const int r1 = r0 + t - 1;
      const int rows_here = (r1 / vho) * hp + (r1 % vho) * vstride - r0 * vstride + kh;
      if (rows_here > pr) pr = rows_here;
    }
    return pr;
  };
  // Largest wave tile first; a candidate must keep three quarters of its pixel capacity busy, fit
  // its patch into the buffer and leave every compute unit a workgroup.
  for (int fp = 4; fp >= 1; fp >>= 1) {
    if (hint_fp && hint_fp != fp) continue;
    if (!has_kernel(g.taps, g.cps, fp, wn)) continue;
    // 1x1 layers: the 256-pixel x 128-channel tile is the dense layer's best (845 against 717 TFLOP/s on a
    // 4096 x 4096 x 8192 product) but takes a gated layer's listed pixels 128 at a pass (measured slower)
    if (g.taps == 1 && fp == 4 && wn == 2 && d.c_base < d.c_in && !hint_fp) continue;
    const TileCfgSize c = tile_cfg_size(g.taps, g.cps, fp, wn);
    if (c.nb < 2) continue;
    int tr = c.bm / vwo;
    if (tr < 1) continue;
    if (tr > rows) tr = (int)rows;
    int t = tr;
    while (t >= 1 && (long long)patch_rows(t) * P * 16 * g.cps > c.pbm) --t;
    if (t < 1) continue;
    const long long wgs = ((rows + t - 1) / t) * g.n_cb;
    if (!hint_fp && fp > 1) {
      if (4 * t * vwo < 3 * c.bm && rows > t) continue;
      if (wgs < n_cu) continue;
    }
    g.fp = fp;
    g.tr = t;
    g.pr = patch_rows(t);
    g.n16 = g.pr * P * g.cps;
    g.hp = hp;
    g.lds_bytes = (size_t)c.lds;
    g.nb = c.nb;
    g.stages[0] = bchunks / g.cps;
    g.stages[1] = cchunks / g.cps;
    g.wpk_stage_bytes = (size_t)c.wbp;
    g.wpk_base_bytes = (size_t)g.n_cb * g.stages[0] * c.wbp;
    g.wpk_cond_bytes = (size_t)g.n_cb * g.stages[1] * c.wbp;
    g.xcd_cb = (g.n_cb % 8 == 0 && (long long)g.taps * d.c_in * d.c_out > (long long)d.n_max * d.h * d.w * d.c_in) ? 1 : 0;
    g.ok = 1;
    return g;
  }
  return g;
}
}  // namespace

TilePlan tile_plan(const cg_conv_desc& d, int n_cu) {
  const int hint_wn = (d.tile_hint >> 4) & 15;
  if (hint_wn) return plan_wn(d, n_cu, hint_wn == 2 ? 2 : 1);
  const TilePlan wide = plan_wn(d, n_cu, 2);
  if (wide.ok) return wide;
  return plan_wn(d, n_cu, 1);
}

hipError_t launch_tile_pack(const TilePlan& g, const Params& p, void* wpk_base, void* wpk_cond, hipStream_t s) {
  const TileCfgSize c = tile_cfg_size(g.taps, g.cps, g.fp, g.wn);
  for (int ph = 0; ph < 2; ++ph) {
    if (g.stages[ph] == 0) continue;
    const long long total = (long long)g.n_cb * g.stages[ph] * (c.wbp / 16);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_tile_kernel, dim3(blocks), dim3(256), 0, s, (const char*)(ph ? p.w_cond : p.w_base),
                       (char*)(ph ? wpk_cond : wpk_base), ph ? p.c_cond : p.c_base, g.elem_bytes, g.ch, g.cps, g.taps,
                       g.bn, c.ks, c.wbp, g.stages[ph], total, g.grp_mode == 2 ? 1 : 0, ph, p.c_base, p.cpg);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_tile(const TilePlan& g, const Params& p, const void* w0, const void* w1, hipStream_t s) {
  const TileGeo q = make_geo(g, p);
  if (p.in_dtype == CG_BF16)
    return g.taps == 9 ? launch_tile_bf16_k3(g, q, p, w0, w1, s) : launch_tile_bf16_k1(g, q, p, w0, w1, s);
  return g.taps == 9 ? launch_tile_i8_k3(g, q, p, w0, w1, s) : launch_tile_i8_k1(g, q, p, w0, w1, s);
}

}  // namespace cg
