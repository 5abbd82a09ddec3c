// Sizes of a configuration of the large-tile kernel, shared by the kernel template and the host plan.
#pragma once

namespace cg {

struct TileCfgSize {
  int bm, bn, ks, kw, wbp, kp, pbm, lps, sz, tab, nb, lds;
};

// taps 9 | 1; cps = 16-byte channel chunks per pixel per stage; fp = 32-pixel fragments per wavefront;
// wn = wavefronts across the channels.  nb = stage buffers: as many (at most four) as 160 KB of LDS and
// the six-bit load counter allow; 0 if not even two fit.
constexpr TileCfgSize tile_cfg_size(int taps, int cps, int fp, int wn) {
  TileCfgSize c{};
  const int wm = 4 / wn;
  c.bn = 64 * wn;
  c.bm = 32 * fp * wm;
  c.ks = (taps * cps + 1) / 2;
  c.kw = (c.ks * 32 * c.bn + 4095) / 4096;
  c.wbp = c.kw * 4096;
  c.kp = (c.bm * 16 * cps * (taps == 1 ? 2 : 3) / 2 + 4095) / 4096;
  c.pbm = c.kp * 4096;
  c.lps = c.kp + c.kw;
  c.sz = c.pbm + c.wbp;
  // after the last stage a buffer carries a 32-row slice of the R tile or the four wavefronts' output tiles
  const int after = 32 * (c.bn * 4 + 16) > 4 * 32 * 144 ? 32 * (c.bn * 4 + 16) : 4 * 32 * 144;
  if (c.sz < after) c.sz = (after + 1023) / 1024 * 1024;
  c.tab = c.bm * (4 + 4 + 2 + 4 * (c.bn / 32)) + 8 * c.bn * 4;
  c.nb = 0;
  for (int nb = 4; nb >= 2; --nb) {
    if (nb * c.sz + c.tab <= 160 * 1024 && (nb - 2) * c.lps <= 63) {
      c.nb = nb;
      break;
    }
  }
  c.lds = c.nb * c.sz + c.tab;
  return c;
}

}  // namespace cg
