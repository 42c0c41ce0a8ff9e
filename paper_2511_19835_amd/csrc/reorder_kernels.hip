// Token reordering around the layer (paper appendix "Implementations": the token sequence is
// reordered before inference so that a block holds spatially close tokens). The order built
// here is the tile order of tile_geom.hpp; text tokens keep their place after the video
// tokens. direction 0 gathers raster-ordered rows into tile order (before the layer),
// direction 1 scatters tile-ordered rows back to raster order (after it).
//
// Pure data movement: every row of d bf16 values is read once and written once, 16 bytes per
// thread, so the kernel is bound by HBM (4 B moved per element). A tile row of tw tokens is
// contiguous on both sides (tw * d * 2 bytes = 2 KB at tw = 8, d = 128).
#include "rsa_common.hpp"
#include "tile_geom.hpp"

namespace rsa {
namespace {

__global__ __launch_bounds__(256) void reorder_kernel(Dims dm, TileGeom g, int direction,
                                                      const uint16_t* __restrict__ src, uint16_t* __restrict__ dst) {
  const int cpr = dm.d / 8;                                   // 16-byte chunks per row
  const int64_t chunks = dm.t * cpr;
  const int bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / dm.heads) * dm.sb + (int64_t)(bh % dm.heads) * dm.sh;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < chunks; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t pos = i / cpr;                              // position in tile order (video) / token index (text)
    const int c = (int)(i % cpr);
    const int64_t ras = pos < dm.tv ? raster_token_of_position(g, (int)pos) : pos;
    const int64_t from = direction == 0 ? ras : pos, to = direction == 0 ? pos : ras;
    const uint4 v = *reinterpret_cast<const uint4*>(src + base + from * dm.st + 8 * c);
    *reinterpret_cast<uint4*>(dst + base + to * dm.st + 8 * c) = v;
  }
}

}  // namespace

hipError_t launch_reorder(const Dims& dm, const int* grid, const int* tile, int direction, const uint16_t* src,
                          uint16_t* dst, hipStream_t s) {
  const TileGeom g = make_tile_geom(grid, tile, 0);
  const int64_t chunks = dm.t * (dm.d / 8);
  int64_t gx = (chunks + 255) / 256;
  if (gx > 8192) gx = 8192;                                   // grid-stride beyond: 32 workgroups per CU and head
  hipLaunchKernelGGL(reorder_kernel, dim3((unsigned)gx, dm.batch * dm.heads), dim3(256), 0, s, dm, g, direction, src, dst);
  return hipGetLastError();
}

}  // namespace rsa
