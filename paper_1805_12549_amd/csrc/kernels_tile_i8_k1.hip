// Instantiations of the large-tile kernel: int8, 1x1.
#include "tile_kernel.h"

namespace cg {

hipError_t launch_tile_i8_k1(const TilePlan& g, const TileGeo& q, const Params& p, const void* w0, const void* w1,
                             hipStream_t s) {
  using namespace tile;
  using Tr = I8Tile;
  if (g.cps == 8 && g.fp == 4 && g.wn == 1)
    return launch_tile_one<Tr, 1, 8, 4, 1, tile_cfg_size(1, 8, 4, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 8 && g.fp == 2 && g.wn == 1)
    return launch_tile_one<Tr, 1, 8, 2, 1, tile_cfg_size(1, 8, 2, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 8 && g.fp == 1 && g.wn == 1)
    return launch_tile_one<Tr, 1, 8, 1, 1, tile_cfg_size(1, 8, 1, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 8 && g.fp == 4 && g.wn == 2)
    return launch_tile_one<Tr, 1, 8, 4, 2, tile_cfg_size(1, 8, 4, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 8 && g.fp == 2 && g.wn == 2)
    return launch_tile_one<Tr, 1, 8, 2, 2, tile_cfg_size(1, 8, 2, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 8 && g.fp == 1 && g.wn == 2)
    return launch_tile_one<Tr, 1, 8, 1, 2, tile_cfg_size(1, 8, 1, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 4 && g.wn == 1)
    return launch_tile_one<Tr, 1, 4, 4, 1, tile_cfg_size(1, 4, 4, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 2 && g.wn == 1)
    return launch_tile_one<Tr, 1, 4, 2, 1, tile_cfg_size(1, 4, 2, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 1 && g.wn == 1)
    return launch_tile_one<Tr, 1, 4, 1, 1, tile_cfg_size(1, 4, 1, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 4 && g.wn == 2)
    return launch_tile_one<Tr, 1, 4, 4, 2, tile_cfg_size(1, 4, 4, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 2 && g.wn == 2)
    return launch_tile_one<Tr, 1, 4, 2, 2, tile_cfg_size(1, 4, 2, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 4 && g.fp == 1 && g.wn == 2)
    return launch_tile_one<Tr, 1, 4, 1, 2, tile_cfg_size(1, 4, 1, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 2 && g.fp == 2 && g.wn == 1)
    return launch_tile_one<Tr, 1, 2, 2, 1, tile_cfg_size(1, 2, 2, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 2 && g.fp == 1 && g.wn == 1)
    return launch_tile_one<Tr, 1, 2, 1, 1, tile_cfg_size(1, 2, 1, 1).nb>(g, q, p, w0, w1, s);
  if (g.cps == 2 && g.fp == 2 && g.wn == 2)
    return launch_tile_one<Tr, 1, 2, 2, 2, tile_cfg_size(1, 2, 2, 2).nb>(g, q, p, w0, w1, s);
  if (g.cps == 2 && g.fp == 1 && g.wn == 2)
    return launch_tile_one<Tr, 1, 2, 1, 2, tile_cfg_size(1, 2, 1, 2).nb>(g, q, p, w0, w1, s);
  return hipErrorInvalidValue;
}

}  // namespace cg
