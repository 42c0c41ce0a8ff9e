// Gain-Aware Pooling Rectification gate (paper Sec. 4.2; Alg. 1 steps 9-11).
//
// The relaxed condition as printed compares |sum_ij s^pool| with |sum_ij Delta s|, and the
// signed double sum of the first-order Delta s is identically zero (block means are
// subtracted). The gate therefore takes the absolute value per term, as the paper's
// un-relaxed definitions of gain and error do, on the two first-order pieces separately:
//     DA[n][m] = mean_{i in block n} |(q_i - q^pool_n) . k^pool_m| * scale
//     DB[n][m] = mean_{j in block m} |q^pool_n . (k_j - k^pool_m)| * scale
//     M_c[n][m] = |s^pool[n][m]| > DA[n][m] + DB[n][m]
// (gain and error both divided by c_n c_m). Each deviation is a skinny GEMM of a token
// block against all pooled vectors of the other side, so the cost is tokens x blocks x d.
//
// deviation_kernel: one workgroup per token block; every wave keeps the whole block as the
// MFMA A operand in registers and walks the pooled vectors 32 at a time. The pooled
// operand is rounded to bf16; accumulation is fp32. The block mean of the products is
// taken from the same accumulators, so the subtraction gives (x_i - mean_i x_i) . p_bf16
// exactly up to fp32 rounding and the only approximation left is p_bf16 for p: a relative
// error of ~1e-3 per product with random sign, ~1e-4 after the mean over the block's rows,
// an order of magnitude inside the band in which the gate is allowed to differ.
#include "rsa_common.hpp"

namespace rsa {
namespace {

template <int D, int BLK>
__global__ __launch_bounds__(256, 2) void deviation_kernel(Dims dm, const uint16_t* __restrict__ X,
                                                           int n_blocks_x,
                                                           const uint16_t* __restrict__ PB,
                                                           int n_other, float* __restrict__ out) {
  constexpr int MT = BLK / 32, KS = D / 16;
  const int xb = blockIdx.x, bh = blockIdx.y;
  const int b = bh / dm.heads, h = bh % dm.heads;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int count = dm.block_count(xb);
  const int64_t t0 = dm.block_start(xb);
  const uint16_t* Xb = X + (int64_t)b * dm.sb + (int64_t)h * dm.sh;

  bf16x8 areg[MT][KS];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int row = 32 * t + l32;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row < count) v = *reinterpret_cast<const uint4*>(Xb + (t0 + row) * dm.st + 16 * s + 8 * hf);
      areg[t][s] = __builtin_bit_cast(bf16x8, v);
    }
  }
  const float inv_c = 1.0f / (float)count;
  float* orow = out + ((size_t)bh * n_blocks_x + xb) * n_other;

  for (int o0 = 32 * wave; o0 < n_other; o0 += 128) {
    const int o = o0 + l32;
    const bool ovalid = o < n_other;
    const uint16_t* prow = PB + ((size_t)bh * n_other + (ovalid ? o : 0)) * D + 8 * hf;
    floatx16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      uint4 vb = make_uint4(0, 0, 0, 0);
      if (ovalid) vb = *reinterpret_cast<const uint4*>(prow + 16 * s);
      const bf16x8 bop = __builtin_bit_cast(bf16x8, vb);
#pragma unroll
      for (int t = 0; t < MT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[t][s], bop, acc[t], 0, 0, 0);
    }
    // accumulator register r of tile t holds row 32t + 8(r/4) + 4*hf + r%4, column l32
    float cs = 0.f;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) cs += acc[t][r];   // rows past the block end are exact zeros
    cs += __shfl_xor(cs, 32);
    const float mean = cs * inv_c;
    float dv = 0.f;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * t + 8 * (r / 4) + 4 * hf + (r % 4);
        dv += (row < count) ? fabsf(acc[t][r] - mean) : 0.f;
      }
    dv += __shfl_xor(dv, 32);
    if (hf == 0 && ovalid) orow[o] = dv * inv_c * dm.scale;
  }
}

// M_c bits from Spool, DA [N][M] and DBt [M][N]; 32 x 32 tiles, DBt transposed through LDS.
__global__ __launch_bounds__(256) void gate_kernel(Dims dm, GaprArgs a) {
  __shared__ float tile[32][33];
  const int bh = blockIdx.z;
  const int m0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
  const float* DBt = a.DBt + (size_t)bh * dm.m * dm.n;
  const float* DA = a.DA + (size_t)bh * dm.n * dm.m;
  const float* S = a.Spool + (size_t)bh * dm.n * dm.m;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int mm = m0 + ty + 8 * it, nn = n0 + tx;
    tile[ty + 8 * it][tx] = (mm < dm.m && nn < dm.n) ? DBt[(size_t)mm * dm.n + nn] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int noff = ty + 8 * it;
    const int nn = n0 + noff, mm = m0 + tx;
    bool pred = false;
    if (nn < dm.n && mm < dm.m) {
      const size_t idx = (size_t)nn * dm.m + mm;
      pred = fabsf(S[idx]) > DA[idx] + tile[tx][noff];
    }
    const unsigned long long bal = __ballot(pred);
    if (tx == 0 && nn < dm.n) {
      const uint32_t word = (threadIdx.x & 32) ? (uint32_t)(bal >> 32) : (uint32_t)bal;
      a.Mc_bits[((size_t)bh * dm.n + nn) * dm.w + blockIdx.x] = word;
    }
  }
}

__global__ void fill_bits_kernel(Dims dm, uint32_t* bits, uint32_t value) {
  const size_t total = (size_t)dm.batch * dm.heads * dm.n * dm.w;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int wd = (int)(i % dm.w);
    uint32_t v = value;
    const int valid = dm.m - wd * 32;
    if (valid < 32) v &= (valid <= 0) ? 0u : ((1u << valid) - 1u);
    bits[i] = v;
  }
}

template <int D, int BLK>
hipError_t launch_gapr_t(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  hipLaunchKernelGGL((deviation_kernel<D, BLK>), dim3(dm.n, bh), dim3(256), 0, s, dm, a.Q, dm.n, a.Kpb, dm.m, a.DA);
  hipLaunchKernelGGL((deviation_kernel<D, BLK>), dim3(dm.m, bh), dim3(256), 0, s, dm, a.K, dm.m, a.Qpb, dm.n, a.DBt);
  hipLaunchKernelGGL(gate_kernel, dim3(dm.w, (dm.n + 31) / 32, bh), dim3(256), 0, s, dm, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gapr(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  if (a.mode != 1) {
    hipLaunchKernelGGL(fill_bits_kernel, dim3(256), dim3(256), 0, s, dm, a.Mc_bits, a.mode == 2 ? 0xffffffffu : 0u);
    return hipGetLastError();
  }
  if (dm.d == 128 && dm.blk == 128) return launch_gapr_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_gapr_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_gapr_t<64, 128>(dm, a, s);
  return launch_gapr_t<64, 64>(dm, a, s);
}

}  // namespace rsa
