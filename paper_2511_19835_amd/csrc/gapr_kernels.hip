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
// deviation_kernel: one workgroup per token block. The block is read once (on the key side the
// launch pools it as well: the only pass over K of the whole preparation), centred on its
// pooled vector (x_i - x^pool, fp32 subtraction, rounded to fp16) and parked in LDS; every
// wave then walks the pooled vectors of the other side 32 at a time against the whole centred
// block (the MFMA A operand, read from LDS just ahead of each MFMA), so the accumulators hold
// the deviations themselves and the epilogue is one |.|-add per element. Three waves per SIMD.
// The key side runs first and leaves DB transposed ([M][N]) in the workspace; the query side runs second
// and never stores DA: it decides the bits of M_c from its registers, S[n][m] and DBt[m][n].
// Measured at the benchmark shape: 0.64 ms per side, 0.52 ms with the pooled-operand loads
// switched off (they are 8 KB from L2 per 32 MFMAs and wave), 0.36 ms of MFMA time at the
// clock the chip holds; a resident copy of the block in registers at two waves per SIMD: 0.65. The pooled operand is rounded to
// fp16 as well; accumulation is fp32. fp16 rather than bf16 because both operands are O(1)
// quantities whose 2^-12 relative rounding leaves DA / DB within 2e-4 relative of fp64
// arithmetic (bf16 operands: up to 1.5e-3, wider than the 1e-3 band in which the gate may
// differ); the MFMA rate is the same. Conversions saturate at the largest finite half.
#include "rsa_common.hpp"

namespace rsa {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#ifndef RSA_DEV_NT
#define RSA_DEV_NT 256
#endif

// 16-byte chunk c of row r sits at chunk position c ^ key(r): 16 consecutive rows read at one
// logical chunk index then touch every LDS bank once. CPR = chunks per row (8 or 16).
template <int CPR>
__device__ __forceinline__ int swizzled(int r, int c) { return r * CPR + (c ^ ((r / (16 / CPR)) & (CPR - 1))); }

#ifndef RSA_DEV_OCC
#define RSA_DEV_OCC 3
#endif
// GATE: the launch for the query side, run second. Its deviations DA[n][.] never leave the registers:
// with the pooled score S[n][m] and the key-side deviation DBt[m][n] of the first launch (one word each
// per lane and iteration, asked for at the start of the iteration) the lane decides its bit of M_c, and
// a ballot makes the mask word of the iteration.
// POOL (key side only): the launch also makes the pooled vector of its block -- it holds the whole block in
// registers before it centres it -- and writes it (fp32, and the fp16 operand copy) for the kernels that
// follow, with the arithmetic of pool_qk_kernel (same thread-to-row mapping, same order of additions), so
// the separate pooling pass over K is not needed.
template <int D, int BLK, int NT, bool GATE, bool POOL>
__global__ __launch_bounds__(NT, RSA_DEV_OCC) void deviation_kernel(Dims dm, const uint16_t* __restrict__ X,
                                                           const float* __restrict__ Xpool, float* __restrict__ Xpool_out,
                                                           uint16_t* __restrict__ Xpool_f16_out, int n_blocks_x,
                                                           const uint16_t* __restrict__ PB,
                                                           int n_other, float* __restrict__ out,
                                                           const float* __restrict__ Spool,
                                                           const float* __restrict__ DBt,
                                                           uint32_t* __restrict__ Mc_bits) {
  constexpr int MT = BLK / 32, KS = D / 16, CPR = D / 8;
  constexpr int NW = NT / 64;                    // waves per workgroup
  constexpr int RPP = NT / CPR;                  // rows staged per pass of the workgroup
  __shared__ u32x4 atile[BLK * CPR];
  // Workgroup i runs on XCD i % 8. Each XCD takes a contiguous eighth of the (batch, head, block)
  // range, so that token blocks that are neighbours run on the same XCD at about the same time: the
  // query side reads DBt[m][n] for a fixed n, 32 neighbouring n to a 128-byte line, which then
  // comes into one L2 once instead of into all eight.
  const int total = n_blocks_x * dm.batch * dm.heads;
  const int xcd = blockIdx.x % 8, q8 = total / 8, r8 = total % 8;
  const int item = xcd * q8 + (xcd < r8 ? xcd : r8) + (int)blockIdx.x / 8;
  const int xb = item % n_blocks_x, bh = item / n_blocks_x;
  const int b = bh / dm.heads, h = bh % dm.heads;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int count = dm.block_count(xb);
  const int64_t t0 = dm.block_start(xb);
  const uint16_t* Xb = X + (int64_t)b * dm.sb + (int64_t)h * dm.sh;

  // ---- stage the centred block: thread -> chunk column tid % CPR, rows tid / CPR + RPP*i ----
  {
    const int cc = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
    u32x4 raw[BLK / RPP];
#pragma unroll
    for (int i = 0; i < BLK / RPP; ++i) {
      const int r = r0 + RPP * i;
      const int rr = r < count ? r : count - 1;                  // stay inside the tensor; zeroed below
      raw[i] = *reinterpret_cast<const u32x4*>(Xb + (t0 + rr) * dm.st + 8 * cc);
    }
    floatx4 m0, m1;
    if constexpr (POOL) {
      static_assert(NT == 256 && RPP * D * 4 <= BLK * CPR * 16, "the mapping of pool_qk_kernel; its partial sums fit the tile");
      __shared__ __align__(16) float mean_lds[D];
      float (*red)[D] = reinterpret_cast<float (*)[D]>(atile);   // the tile is written after the sums have been read
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < BLK / RPP; ++i) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r0 + RPP * i < count) v = make_uint4(raw[i].x, raw[i].y, raw[i].z, raw[i].w);
        accumulate8(acc, v);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) red[r0][cc * 8 + e] = acc[e];
      __syncthreads();
      if (threadIdx.x < D) {
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r) sum += red[r][threadIdx.x];
        const float mean = sum / (float)count;
        mean_lds[threadIdx.x] = mean;
        Xpool_out[((size_t)bh * n_blocks_x + xb) * D + threadIdx.x] = mean;
        Xpool_f16_out[(size_t)bh * gate_operand_vectors(n_blocks_x) * D + gate_operand_offset<D>(xb, threadIdx.x)] = to_f16_bits_sat(mean);
      }
      __syncthreads();
      m0 = *reinterpret_cast<const floatx4*>(mean_lds + 8 * cc);
      m1 = *reinterpret_cast<const floatx4*>(mean_lds + 8 * cc + 4);
      __syncthreads();                                             // every read of the sums is done
    } else {
      const float* mp = Xpool + ((size_t)bh * n_blocks_x + xb) * D + 8 * cc;
      m0 = *reinterpret_cast<const floatx4*>(mp);
      m1 = *reinterpret_cast<const floatx4*>(mp + 4);
    }
#pragma unroll
    for (int i = 0; i < BLK / RPP; ++i) {
      const int r = r0 + RPP * i;
      u32x4 c;
      c.x = pack_f16x2_sat(bf16_bits_to_float(raw[i].x & 0xffffu) - m0[0], bf16_bits_to_float(raw[i].x >> 16) - m0[1]);
      c.y = pack_f16x2_sat(bf16_bits_to_float(raw[i].y & 0xffffu) - m0[2], bf16_bits_to_float(raw[i].y >> 16) - m0[3]);
      c.z = pack_f16x2_sat(bf16_bits_to_float(raw[i].z & 0xffffu) - m1[0], bf16_bits_to_float(raw[i].z >> 16) - m1[1]);
      c.w = pack_f16x2_sat(bf16_bits_to_float(raw[i].w & 0xffffu) - m1[2], bf16_bits_to_float(raw[i].w >> 16) - m1[3]);
      if (r >= count) c = u32x4{0u, 0u, 0u, 0u};                // rows past a ragged block contribute nothing
      atile[swizzled<CPR>(r, cc)] = c;
    }
  }
  __syncthreads();
  // the A operand of an MFMA is read from LDS just ahead of it: the registers that a resident copy
  // of the block would take (128 at d = 128) buy a third wave per SIMD instead
  const u32x4* arow[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) arow[t] = atile + (32 * t + l32) * CPR;
  const int akey = (l32 / (16 / CPR)) & (CPR - 1);
#define RSA_DEV_A(t, s) __builtin_bit_cast(halfx8, arow[t][(2 * (s) + hf) ^ akey])

  const float outscale = dm.scale / (float)count;
  float* orow = out + ((size_t)bh * n_blocks_x + xb) * n_other;
  // pooled vectors of the other side, fp16, in the layout of gate_operand_offset: the 32 vectors
  // of one iteration and one k-step are 1 KB in a row, 16 bytes per lane
  const uint16_t* PBh = PB + (size_t)bh * gate_operand_vectors(n_other) * D + 8 * lane;

  // The B operand of one iteration is 32 pooled vectors: lane (l32, hf) supplies channels
  // 16s + 8hf .. +7 of vector o0 + l32 for k-step s. It is fetched a whole iteration ahead
  // (two register sets that swap roles); to make room the block's row tiles are taken two at
  // a time, so only 32 accumulator registers are live. Vectors past the end of the last group
  // are padding: they only feed output columns that are never stored.
  constexpr int TP = MT < 2 ? MT : 2;
  auto load_vectors = [&](u32x4 (&dstv)[KS], int o0) __attribute__((always_inline)) {
    const uint16_t* p = PBh + (size_t)(o0 / 32) * KS * 512;
#pragma unroll
    for (int s = 0; s < KS; ++s) dstv[s] = *reinterpret_cast<const u32x4*>(p + 512 * s);
  };
  auto iteration = [&](const u32x4 (&bv)[KS], u32x4 (&bnext)[KS], int o0) __attribute__((always_inline)) {
    if (o0 + 32 * NW < n_other) load_vectors(bnext, o0 + 32 * NW);
    float s_val = 0.f, db_val = 0.f;
    if constexpr (GATE) {
      const int m = o0 + l32 < n_other ? o0 + l32 : n_other - 1;
      s_val = Spool[((size_t)bh * n_blocks_x + xb) * n_other + m];
      db_val = DBt[((size_t)bh * n_other + m) * n_blocks_x + xb];
    }
    asm volatile("" ::: "memory");      // the A operand is re-read every iteration: no hoisting into registers
    // every accumulator of a lane belongs to column o0 + l32; its rows are spread over the
    // registers, the row tiles and the two half-waves
    float dv4[4] = {0.f, 0.f, 0.f, 0.f};       // four partial sums: no long chain of dependent adds
#pragma unroll
    for (int t0 = 0; t0 < MT; t0 += TP) {
      floatx16 acc[TP];
#pragma unroll
      for (int t = 0; t < TP; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int t = 0; t < TP; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(RSA_DEV_A(t0 + t, s), __builtin_bit_cast(halfx8, bv[s]), acc[t], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < TP; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) dv4[r % 4] += fabsf(acc[t][r]);
    }
    float dv = (dv4[0] + dv4[1]) + (dv4[2] + dv4[3]);
    dv += __shfl_xor(dv, 32);
    if constexpr (GATE) {
      const bool pred = o0 + l32 < n_other && fabsf(s_val) > dv * outscale + db_val;
      const unsigned long long word = __ballot(pred);
      if (lane == 0) Mc_bits[((size_t)bh * n_blocks_x + xb) * dm.w + o0 / 32] = (uint32_t)word;
    } else {
      if (hf == 0 && o0 + l32 < n_other) orow[o0 + l32] = dv * outscale;
    }
  };
  u32x4 b0[KS], b1[KS];
  if (32 * wave < n_other) load_vectors(b0, 32 * wave);
  for (int o0 = 32 * wave; o0 < n_other; o0 += 64 * NW) {
    iteration(b0, b1, o0);
    if (o0 + 32 * NW < n_other) iteration(b1, b0, o0 + 32 * NW);
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
hipError_t launch_gapr_keys_t(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  constexpr int NT = RSA_DEV_NT;
  // DBt [M][N] to the workspace
  if (a.Kp_out)
    hipLaunchKernelGGL((deviation_kernel<D, BLK, NT, false, true>), dim3(dm.m * bh), dim3(NT), 0, s, dm, a.K, nullptr, a.Kp_out,
                       a.Kpb_out, dm.m, a.Qpb, dm.n, a.DBt, nullptr, nullptr, nullptr);
  else
    hipLaunchKernelGGL((deviation_kernel<D, BLK, NT, false, false>), dim3(dm.m * bh), dim3(NT), 0, s, dm, a.K, a.Kp, nullptr,
                       nullptr, dm.m, a.Qpb, dm.n, a.DBt, nullptr, nullptr, nullptr);
  return hipGetLastError();
}
template <int D, int BLK>
hipError_t launch_gapr_queries_t(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  constexpr int NT = RSA_DEV_NT;
  // turns its deviations into the bits of M_c on the spot
  hipLaunchKernelGGL((deviation_kernel<D, BLK, NT, true, false>), dim3(dm.n * bh), dim3(NT), 0, s, dm, a.Q, a.Qp, nullptr, nullptr,
                     dm.n, a.Kpb, dm.m, nullptr, a.Spool, a.DBt, a.Mc_bits);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gapr_keys(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_gapr_keys_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_gapr_keys_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_gapr_keys_t<64, 128>(dm, a, s);
  return launch_gapr_keys_t<64, 64>(dm, a, s);
}

hipError_t launch_gapr_queries(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_gapr_queries_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_gapr_queries_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_gapr_queries_t<64, 128>(dm, a, s);
  return launch_gapr_queries_t<64, 64>(dm, a, s);
}

hipError_t launch_gapr(const Dims& dm, const GaprArgs& a, hipStream_t s) {
  if (a.mode != 1) {
    hipLaunchKernelGGL(fill_bits_kernel, dim3(256), dim3(256), 0, s, dm, a.Mc_bits, a.mode == 2 ? 0xffffffffu : 0u);
    return hipGetLastError();
  }
  const hipError_t e = launch_gapr_keys(dm, a, s);
  return e != hipSuccess ? e : launch_gapr_queries(dm, a, s);
}

}  // namespace rsa
