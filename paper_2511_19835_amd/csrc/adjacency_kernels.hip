// Adjacency mask M_adja (paper Alg. 1 "Require" and step 14; Sec. 4.3: spatial-temporal
// neighbour blocks are always kept). The paper does not define it further; the reading
// built here: video tokens are stored tile by tile over the (T, H, W) latent grid (tiles in
// raster order, tokens in raster order inside a tile, tiles at the upper faces of the grid
// may be partial); a video query block and a video key block are neighbours when some tile
// touched by one and some tile touched by the other differ by at most `radius` in every tile
// coordinate. Text key blocks are never forced.
//
// Because tiles are stored in raster order, the tokens of block n = [nB, min((n+1)B, T_v))
// touch a contiguous range of raster tile indices, and the first token of tile (a, b, c) has
// a closed form:
//     start(a,b,c) = min(a*tt, T)*H*W + ct(a) * ( min(b*th, H)*W + ch(b) * min(c*tw, W) )
// with ct(a) = min(tt, T - a*tt) and likewise ch, cw. The tile of a token follows by three
// integer divisions. One thread decides one (query block, key block) pair; a ballot packs 32
// decisions into a mask word, written for every (batch, head).
#include "rsa_common.hpp"
#include "tile_geom.hpp"

namespace rsa {
namespace {

__global__ __launch_bounds__(64) void adjacency_kernel(Dims dm, TileGeom g, uint32_t* __restrict__ bits) {
  const int n = blockIdx.y;
  const int m = blockIdx.x * 64 + threadIdx.x;
  bool near = false;
  if (m < dm.n) {
    const int n_lo = n * dm.blk, n_hi = (int)min((int64_t)(n + 1) * dm.blk, dm.tv) - 1;
    const int m_lo = m * dm.blk, m_hi = (int)min((int64_t)(m + 1) * dm.blk, dm.tv) - 1;
    const int fa = raster(g, tile_of_token(g, n_lo)), la = raster(g, tile_of_token(g, n_hi));
    const int fb = raster(g, tile_of_token(g, m_lo)), lb = raster(g, tile_of_token(g, m_hi));
    for (int i = fa; i <= la && !near; ++i) {
      const TileIdx p = unraster(g, i);
      for (int j = fb; j <= lb; ++j) {
        const TileIdx q = unraster(g, j);
        if (abs(p.a - q.a) <= g.radius && abs(p.b - q.b) <= g.radius && abs(p.c - q.c) <= g.radius) {
          near = true;
          break;
        }
      }
    }
  }
  const unsigned long long bal = __ballot(near);
  const int lane = threadIdx.x;
  if (lane == 0 || lane == 32) {
    const int wd = blockIdx.x * 2 + lane / 32;
    if (wd < dm.w) {
      const uint32_t word = lane ? (uint32_t)(bal >> 32) : (uint32_t)bal;
      const int bh = dm.batch * dm.heads;
      for (int i = 0; i < bh; ++i) bits[((size_t)i * dm.n + n) * dm.w + wd] = word;
    }
  }
}

}  // namespace

hipError_t launch_adjacency(const Dims& dm, const int* grid, const int* tile, int radius, uint32_t* bits,
                            hipStream_t s) {
  const TileGeom g = make_tile_geom(grid, tile, radius);
  hipLaunchKernelGGL(adjacency_kernel, dim3((dm.w + 1) / 2, dm.n), dim3(64), 0, s, dm, g, bits);
  return hipGetLastError();
}

}  // namespace rsa
