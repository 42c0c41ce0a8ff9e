// Uniform block pooling of Q, K, V (paper Sec. 3.2 pooled equations; Alg. 1 step 3) and
// the channel-major copy of V that the attention kernel consumes.
//
// HBM-bound streaming reduction: one workgroup per (key block, batch*head, tensor), each
// thread owns one 16-byte column chunk and walks the block's rows with all loads in
// flight before the first add. Algorithmic traffic: 2 bytes read per input element, plus
// 2 bytes written per V element for the channel-major copy.
#include "rsa_common.hpp"
#include "text_mass.hpp"

namespace rsa {
namespace {

// Reduce the per-thread partial sums over the row groups and write the block mean
// (fp32) and, optionally, an fp16 copy (saturated; the gate GEMMs' pooled operand).
template <int D, int RPP>
__device__ inline void finish_mean(float (*red)[D], const float (&acc)[8], int r0, int cc, int count,
                                   float* mean_out, uint16_t* f16_base, int vec) {
#pragma unroll
  for (int e = 0; e < 8; ++e) red[r0][cc * 8 + e] = acc[e];
  __syncthreads();
  const int tid = threadIdx.x;
  if (tid < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPP; ++r) s += red[r][tid];
    const float mean = s / (float)count;
    mean_out[tid] = mean;
    if (f16_base) f16_base[gate_operand_offset<D>(vec, tid)] = to_f16_bits_sat(mean);
  }
}

template <int D, int BLK>
__global__ __launch_bounds__(256) void pool_qk_kernel(Dims dm, PoolArgs a) {
  constexpr int CPR = D / 8;      // 16-byte chunks per row
  constexpr int RPP = 256 / CPR;  // rows per pass
  constexpr int NPASS = BLK / RPP;
  __shared__ float red[RPP][D];
  const int m = blockIdx.x, bh = blockIdx.y, which = blockIdx.z;
  if (which == 0 && m >= dm.n) return;  // pooled queries exist for video blocks only
  const int b = bh / dm.heads, h = bh % dm.heads;
  const uint16_t* X = (which == 0 ? a.Q : a.K) + (int64_t)b * dm.sb + (int64_t)h * dm.sh;
  const int64_t t0 = dm.block_start(m);
  const int count = dm.block_count(m);
  const int cc = threadIdx.x % CPR, r0 = threadIdx.x / CPR;

  uint4 v[NPASS];
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int r = r0 + p * RPP;
    v[p] = make_uint4(0, 0, 0, 0);
    if (r < count) v[p] = *reinterpret_cast<const uint4*>(X + (t0 + r) * dm.st + cc * 8);
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < NPASS; ++p) accumulate8(acc, v[p]);

  if (which == 0) {
    const size_t row = (size_t)bh * dm.n + m;
    finish_mean<D, RPP>(red, acc, r0, cc, count, a.Qp + row * D,
                        a.Qpb ? a.Qpb + (size_t)bh * gate_operand_vectors(dm.n) * D : nullptr, m);
  } else {
    const size_t row = (size_t)bh * dm.m + m;
    finish_mean<D, RPP>(red, acc, r0, cc, count, a.Kp + row * D,
                        a.Kpb ? a.Kpb + (size_t)bh * gate_operand_vectors(dm.m) * D : nullptr, m);
  }
}

// V: block mean plus the channel-major tile Vt[d][BLK]. Position 16c + 8h + 4g + e of a
// channel row holds token 16c + 8g + 4h + e of the block (the two middle groups of four
// swapped in every run of 16), which is the order in which one half-wave holds the
// softmax probabilities after the S^T = K Q^T product; tokens past the block end are 0.
// LDS: 256 / (D/8) rows of D floats for the mean, then BLK rows of D/2 + 1 words for the tile.
template <int D, int BLK>
struct PoolVLds {
  static constexpr int TS = D / 2 + 1;          // tile row stride in 32-bit words (odd: spreads rows over banks)
  static constexpr int RED = (256 / (D / 8)) * D;
  static constexpr int WORDS = RED + BLK * TS;
};
template <int D, int BLK>
__device__ __forceinline__ void pool_v_block(const Dims& dm, const PoolArgs& a, int m, int bh, uint32_t* lds) {
  constexpr int CPR = D / 8;
  constexpr int RPP = 256 / CPR;
  constexpr int NPASS = BLK / RPP;
  constexpr int TS = PoolVLds<D, BLK>::TS;
  float (*red)[D] = reinterpret_cast<float (*)[D]>(lds);
  uint32_t* tile = lds + PoolVLds<D, BLK>::RED;
  const int b = bh / dm.heads, h = bh % dm.heads;
  const uint16_t* X = a.V + (int64_t)b * dm.sb + (int64_t)h * dm.sh;
  const int64_t t0 = dm.block_start(m);
  const int count = dm.block_count(m);
  const int cc = threadIdx.x % CPR, r0 = threadIdx.x / CPR;

  uint4 v[NPASS];
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int r = r0 + p * RPP;
    v[p] = make_uint4(0, 0, 0, 0);
    if (r < count) v[p] = *reinterpret_cast<const uint4*>(X + (t0 + r) * dm.st + cc * 8);
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    accumulate8(acc, v[p]);
    uint32_t* dst = tile + (r0 + p * RPP) * TS + cc * 4;
    dst[0] = v[p].x; dst[1] = v[p].y; dst[2] = v[p].z; dst[3] = v[p].w;
  }
  const size_t row = (size_t)bh * dm.m + m;
  finish_mean<D, RPP>(red, acc, r0, cc, count, a.Vp + row * D, nullptr, 0);  // contains a barrier

  // Each thread emits, for one pair of adjacent channels, 8 consecutive positions.
  uint16_t* out = a.Vt + row * (size_t)D * BLK;
  constexpr int PCS = BLK / 8;                 // 16-byte chunks per channel row
  constexpr int TASKS = (D / 2) * PCS;
  for (int task = threadIdx.x; task < TASKS; task += 256) {
    const int dpair = task / PCS, pc = task % PCS;
    const int kv0 = 16 * (pc >> 1) + 4 * (pc & 1);
    uint32_t w[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = tile[(kv0 + 8 * (e >> 2) + (e & 3)) * TS + dpair];
    uint4 lo, hi;
    lo.x = (w[0] & 0xffffu) | (w[1] << 16); hi.x = (w[0] >> 16) | (w[1] & 0xffff0000u);
    lo.y = (w[2] & 0xffffu) | (w[3] << 16); hi.y = (w[2] >> 16) | (w[3] & 0xffff0000u);
    lo.z = (w[4] & 0xffffu) | (w[5] << 16); hi.z = (w[4] >> 16) | (w[5] & 0xffff0000u);
    lo.w = (w[6] & 0xffffu) | (w[7] << 16); hi.w = (w[6] >> 16) | (w[7] & 0xffff0000u);
    *reinterpret_cast<uint4*>(out + (size_t)(2 * dpair) * BLK + pc * 8) = lo;
    *reinterpret_cast<uint4*>(out + (size_t)(2 * dpair + 1) * BLK + pc * 8) = hi;
  }
}

template <int D, int BLK>
__global__ __launch_bounds__(256) void pool_v_kernel(Dims dm, PoolArgs a) {
  __shared__ uint32_t lds[PoolVLds<D, BLK>::WORDS];
  pool_v_block<D, BLK>(dm, a, blockIdx.x, blockIdx.y, lds);
}

// The same launch with the text log-masses on board: the first `text_wgs` workgroups of every
// (batch, head) take eight pooled queries each against the text keys (vector-ALU work, no traffic to
// speak of), the others pool a block of V (HBM-bound) -- the one hides under the other.
template <int D, int BLK>
__global__ __launch_bounds__(256) void pool_v_text_kernel(Dims dm, PoolArgs a, ScoreArgs sa, int text_wgs) {
  constexpr int WORDS = PoolVLds<D, BLK>::WORDS > text_mass_lds_floats<D>() ? PoolVLds<D, BLK>::WORDS : text_mass_lds_floats<D>();
  __shared__ uint32_t lds[WORDS];
  if ((int)blockIdx.x < text_wgs) {          // the whole workgroup
    text_mass_block<D, BLK>(dm, sa, blockIdx.x * kTextMassQueries, blockIdx.y, reinterpret_cast<float*>(lds));
    return;
  }
  pool_v_block<D, BLK>(dm, a, (int)blockIdx.x - text_wgs, blockIdx.y, lds);
}

template <int D, int BLK>
hipError_t launch_pool_t(const Dims& dm, const PoolArgs& a, hipStream_t s) {
  const dim3 block(256);
  if (a.Q && a.K)    // values only: the caller keeps the pooled queries / keys of an earlier call
    hipLaunchKernelGGL((pool_qk_kernel<D, BLK>), dim3(dm.m, dm.batch * dm.heads, a.skip_k ? 1 : 2), block, 0, s, dm, a);
  if (a.text_K && a.text_Lmass && a.Q && dm.tt > 0) {   // Qp is written by the launch above
    ScoreArgs sa = {};
    sa.K = a.text_K; sa.Qp = a.Qp; sa.Lmass = a.text_Lmass;
    const int text_wgs = (dm.n + kTextMassQueries - 1) / kTextMassQueries;
    hipLaunchKernelGGL((pool_v_text_kernel<D, BLK>), dim3(dm.m + text_wgs, dm.batch * dm.heads, 1), block, 0, s, dm, a, sa, text_wgs);
  } else {
    hipLaunchKernelGGL((pool_v_kernel<D, BLK>), dim3(dm.m, dm.batch * dm.heads, 1), block, 0, s, dm, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_pool(const Dims& dm, const PoolArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_pool_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_pool_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_pool_t<64, 128>(dm, a, s);
  return launch_pool_t<64, 64>(dm, a, s);
}

}  // namespace rsa
