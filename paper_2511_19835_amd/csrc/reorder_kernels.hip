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

// A wave owns 64 consecutive positions: lane L works out where position p0 + L lives in raster
// order (the integer divisions are done once per row, not once per 16-byte chunk), then the
// wave moves the 64 rows 64/cpr at a time, fetching each row's source from the lane that
// computed it. All cpr loads of a lane are independent and in flight together.
template <int CPR>
__global__ __launch_bounds__(256) void reorder_kernel(Dims dm, TileGeom g, int direction,
                                                      const uint16_t* __restrict__ src, uint16_t* __restrict__ dst) {
  constexpr int RPI = 64 / CPR;                               // rows per load instruction of a wave
  const int lane = threadIdx.x % 64;
  const int bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / dm.heads) * dm.sb + (int64_t)(bh % dm.heads) * dm.sh;
  const int64_t waves = (int64_t)gridDim.x * (blockDim.x / 64);
  const int c = lane % CPR, sub = lane / CPR;
  for (int64_t p0 = (blockIdx.x * (int64_t)(blockDim.x / 64) + threadIdx.x / 64) * 64; p0 < dm.t; p0 += waves * 64) {
    const int64_t pos = p0 + lane;
    int ras = (int)pos;                                       // text rows and rows past the end: identity
    if (pos < dm.tv) ras = raster_token_of_position(g, (int)pos);
    uint4 v[CPR];
#pragma unroll
    for (int j = 0; j < CPR; ++j) {
      const int r = j * RPI + sub;                            // row of this lane in the wave's 64
      const int64_t rp = p0 + r;
      const int64_t rr = __shfl(ras, r);
      const int64_t from = direction == 0 ? rr : rp;
      v[j] = make_uint4(0, 0, 0, 0);
      if (rp < dm.t) v[j] = *reinterpret_cast<const uint4*>(src + base + from * dm.st + 8 * c);
    }
#pragma unroll
    for (int j = 0; j < CPR; ++j) {
      const int r = j * RPI + sub;
      const int64_t rp = p0 + r;
      const int64_t rr = __shfl(ras, r);
      const int64_t to = direction == 0 ? rp : rr;
      if (rp < dm.t) *reinterpret_cast<uint4*>(dst + base + to * dm.st + 8 * c) = v[j];
    }
  }
}

}  // namespace

hipError_t launch_reorder(const Dims& dm, const int* grid, const int* tile, int direction, const uint16_t* src,
                          uint16_t* dst, hipStream_t s) {
  const TileGeom g = make_tile_geom(grid, tile, 0);
  int64_t gx = (dm.t + 255) / 256;                            // 4 waves x 64 positions per workgroup
  if (gx > 4096) gx = 4096;                                   // grid-stride beyond
  if (dm.d == 128)
    hipLaunchKernelGGL((reorder_kernel<16>), dim3((unsigned)gx, dm.batch * dm.heads), dim3(256), 0, s, dm, g, direction, src, dst);
  else
    hipLaunchKernelGGL((reorder_kernel<8>), dim3((unsigned)gx, dm.batch * dm.heads), dim3(256), 0, s, dm, g, direction, src, dst);
  return hipGetLastError();
}

}  // namespace rsa
