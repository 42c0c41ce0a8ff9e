// Geometry of the tile order of video tokens: the (T, H, W) latent grid is cut into tiles of
// (tt, th, tw); tiles are stored in raster order, tokens in raster order inside a tile; tiles
// at the upper faces of the grid may be partial. The first token of tile (a, b, c) is
//     start(a,b,c) = min(a*tt, T)*H*W + ct(a) * ( min(b*th, H)*W + ch(b) * min(c*tw, W) )
// with ct(a) = min(tt, T - a*tt) and likewise ch, cw.
#pragma once

#include <hip/hip_runtime.h>

namespace rsa {

struct TileGeom {
  int T, H, W;        // latent grid
  int tt, th, tw;     // tile
  int nb, nc;         // tiles along h and w
  int radius;
};

struct TileIdx { int a, b, c; };

__device__ inline TileIdx tile_of_token(const TileGeom& g, int x) {
  TileIdx t;
  const int layer = g.tt * g.H * g.W;                 // tokens of a full layer of tiles
  t.a = x / layer;
  const int ct = min(g.tt, g.T - t.a * g.tt);
  int rem = x - t.a * layer;
  const int strip = ct * g.th * g.W;                  // tokens of a full strip of tiles along w
  t.b = rem / strip;
  const int ch = min(g.th, g.H - t.b * g.th);
  rem -= t.b * strip;
  t.c = rem / (ct * ch * g.tw);
  return t;
}
__device__ inline int raster(const TileGeom& g, TileIdx t) { return (t.a * g.nb + t.b) * g.nc + t.c; }
__device__ inline TileIdx unraster(const TileGeom& g, int r) {
  TileIdx t;
  t.c = r % g.nc;
  r /= g.nc;
  t.b = r % g.nb;
  t.a = r / g.nb;
  return t;
}

// Raster index (t*H + h)*W + w of the video token stored at position x of the tile order.
__device__ inline int raster_token_of_position(const TileGeom& g, int x) {
  const TileIdx t = tile_of_token(g, x);
  const int ct = min(g.tt, g.T - t.a * g.tt), ch = min(g.th, g.H - t.b * g.th), cw = min(g.tw, g.W - t.c * g.tw);
  const int start = min(t.a * g.tt, g.T) * g.H * g.W + ct * (min(t.b * g.th, g.H) * g.W + ch * min(t.c * g.tw, g.W));
  const int local = x - start;                       // raster position inside the (possibly partial) tile
  const int lw = local % cw, lh = (local / cw) % ch, lt = local / (cw * ch);
  return ((t.a * g.tt + lt) * g.H + (t.b * g.th + lh)) * g.W + (t.c * g.tw + lw);
}

inline TileGeom make_tile_geom(const int* grid, const int* tile, int radius) {
  TileGeom g;
  g.T = grid[0]; g.H = grid[1]; g.W = grid[2];
  g.tt = tile[0]; g.th = tile[1]; g.tw = tile[2];
  g.nb = (g.H + g.th - 1) / g.th;
  g.nc = (g.W + g.tw - 1) / g.tw;
  g.radius = radius;
  return g;
}

}  // namespace rsa
