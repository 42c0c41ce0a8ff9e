// Block-sparse flash attention with the rectification fused into the epilogue
// (paper Sec. 3.1 sparse attention, Alg. 1 steps 16-17; Sec. 4.1 / 4.2, Alg. 1 steps 19-23).
//
// One workgroup per (batch*head, query block). Video query blocks walk their compact,
// ascending list of critical key blocks; text query blocks (and every block under
// RSA_DENSE) walk all M key blocks. Per key block the K tile [B][d] and the channel-major
// V tile [d][B] are staged in LDS (rows padded by 16 bytes so a 128-bit operand read by 16
// consecutive lanes touches every bank once) and each wave computes, with
// v_mfma_f32_32x32x16_bf16,
//     S^T = K Q^T      (M = key, N = query, k = channel)      -> accumulators: one query
//     O^T += V^T P^T   (M = channel, N = query, k = key)         column per lane
// so that the online softmax is lane-local except for one exchange between the two
// half-waves, and the probabilities a lane holds after the first product are exactly the
// B operand it needs for the second (the V tile is stored in that key order).
// Epilogue: O = R_n * acc / l + C_n with C_n = sum_{m: not kept and M_c} A^pool[n][m] v^pool_m.
//
// MFMA-bound by design: 4*B*B*d flop per (query block, key block) pair against 2*B*d*2
// bytes of K/V tile traffic that is meant to come from L2 / Infinity Cache: workgroups that
// run at the same time work on neighbouring query blocks of the same head, and each XCD
// (workgroup id modulo 8) owns a contiguous range of query blocks.
#include "rsa_common.hpp"

namespace rsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

template <int D, int BLK, int QW>
struct AttnCfg {
  static constexpr int NW = BLK / QW;       // waves per workgroup
  static constexpr int NTHR = 64 * NW;
  static constexpr int NT = QW / 32;        // query tiles per wave
  static constexpr int KT = BLK / 32;       // key tiles of S^T
  static constexpr int KS = D / 16;         // k-steps of K Q^T
  static constexpr int DT = D / 32;         // channel tiles of O^T
  static constexpr int KROW = D * 2 + 16;   // bytes per K row in LDS
  static constexpr int VROW = BLK * 2 + 16; // bytes per V^T row in LDS
  static constexpr int LDS_BYTES = BLK * KROW + D * VROW;
};

template <int D, int BLK, int QW>
__global__ __launch_bounds__(64 * BLK / QW) void attn_kernel(Dims dm, AttnArgs a, int n_text_items,
                                                                        int chunk) {
  using C = AttnCfg<D, BLK, QW>;
  __shared__ __attribute__((aligned(16))) unsigned char lds[C::LDS_BYTES];
  __shared__ float comp[2][D];
  unsigned char* ldsK = lds;
  unsigned char* ldsV = lds + BLK * C::KROW;

  // ---- which (batch*head, query block) is this workgroup ---------------------------------
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  int bh, qb;
  {
    const int id = blockIdx.x;
    if (id < n_text_items) {           // long dense rows first
      const int per = dense_all ? dm.m : dm.mt;
      bh = id / per;
      qb = dense_all ? id % per : dm.n + id % per;
    } else {
      const int v = id - n_text_items;
      const int xcd = v & 7, j = v >> 3;
      bh = j / chunk;
      qb = xcd * chunk + j % chunk;
      if (qb >= dm.n) return;
    }
  }
  const int b = bh / dm.heads, h = bh % dm.heads;
  const bool sparse_row = !dense_all && qb < dm.n;
  const size_t vrow = (size_t)bh * dm.n + qb;      // row of the per-video-block tensors
  const int nlist = sparse_row ? a.count[vrow] : dm.m;
  const int32_t* list = sparse_row ? a.block_idx + vrow * dm.m : nullptr;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int64_t base = (int64_t)b * dm.sb + (int64_t)h * dm.sh;
  const uint16_t* Qb = a.Q + base;
  const uint16_t* Kb = a.K + base;
  const uint16_t* Vtb = a.Vt + (size_t)bh * dm.m * D * BLK;

  // ---- pooled compensation C_n (Alg. 1 step 21), parked in LDS for the epilogue ----------
  const bool do_comp = sparse_row && (a.flags & RSA_COMPENSATE);
  if (do_comp) {
    constexpr int G = C::NTHR / D;                 // thread groups striding over mask words
    const int dd = tid % D, g = tid / D;
    float accv = 0.f;
    if (g < 2) {
      const uint32_t* mk = a.mask_bits + vrow * dm.w;
      const uint32_t* mc = a.Mc_bits + vrow * dm.w;
      const float* Ap = a.Apool + vrow * dm.m;
      const float* Vp = a.Vp + (size_t)bh * dm.m * D;
      constexpr int GS = G < 2 ? G : 2;
      for (int wd = g; wd < dm.w; wd += GS) {
        uint32_t bits = ~mk[wd] & mc[wd];
        while (bits) {
          const int bit = __builtin_ctz(bits);
          bits &= bits - 1;
          const int m = wd * 32 + bit;
          accv = fmaf(Ap[m], Vp[(size_t)m * D + dd], accv);
        }
      }
      comp[g][dd] = accv;
    }
    if (G < 2 && tid < D) comp[1][tid] = 0.f;
  }

  // ---- Q as the B operand of S^T = K Q^T, resident in registers --------------------------
  const int q_count = dm.block_count(qb);
  const int64_t q_t0 = dm.block_start(qb);
  bf16x8 qreg[C::NT][C::KS];
#pragma unroll
  for (int nt = 0; nt < C::NT; ++nt) {
    const int q = wave * QW + 32 * nt + l32;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (q < q_count) v = *reinterpret_cast<const uint4*>(Qb + (q_t0 + q) * dm.st + 16 * s + 8 * hf);
      qreg[nt][s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  floatx16 oacc[C::DT][C::NT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][nt][r] = 0.f;
  float mrun[C::NT], lrun[C::NT];
#pragma unroll
  for (int nt = 0; nt < C::NT; ++nt) { mrun[nt] = -INFINITY; lrun[nt] = 0.f; }
  const float cs = dm.scale * kLog2e;

  for (int j = 0; j < nlist; ++j) {
    const int m = list ? list[j] : j;
    const int kv_count = dm.block_count(m);
    const int64_t kv_t0 = dm.block_start(m);
    __syncthreads();  // everyone is done reading the previous tiles
    {
      constexpr int KCH = D / 8;
      const uint16_t* src = Kb + kv_t0 * dm.st;
#pragma unroll 4
      for (int idx = tid; idx < BLK * KCH; idx += C::NTHR) {
        const int r = idx / KCH, cc = idx % KCH;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < kv_count) v = *reinterpret_cast<const uint4*>(src + (int64_t)r * dm.st + cc * 8);
        *reinterpret_cast<uint4*>(ldsK + r * C::KROW + cc * 16) = v;
      }
      constexpr int VCH = BLK / 8;
      const uint16_t* vsrc = Vtb + (size_t)m * D * BLK;
#pragma unroll 4
      for (int idx = tid; idx < D * VCH; idx += C::NTHR) {
        const int dd = idx / VCH, pc = idx % VCH;
        const uint4 v = *reinterpret_cast<const uint4*>(vsrc + dd * BLK + pc * 8);
        *reinterpret_cast<uint4*>(ldsV + dd * C::VROW + pc * 16) = v;
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T ------------------------------------------------------------------
    floatx16 sacc[C::KT][C::NT];
#pragma unroll
    for (int t = 0; t < C::KT; ++t)
#pragma unroll
      for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[t][nt][r] = 0.f;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
#pragma unroll
      for (int t = 0; t < C::KT; ++t) {
        const bf16x8 ka = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(ldsK + (32 * t + l32) * C::KROW + (16 * s + 8 * hf) * 2));
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
          sacc[t][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[nt][s], sacc[t][nt], 0, 0, 0);
      }
    }
    // accumulator register r of key tile t is key 32t + 8(r/4) + 4*hf + r%4 of the block
    if (kv_count < BLK) {
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = 32 * t + 8 * (r / 4) + 4 * hf + (r % 4);
          if (kv >= kv_count) {
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt) sacc[t][nt][r] = -INFINITY;
          }
        }
    }

    // ---- online softmax, one query column per lane -----------------------------------
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt) {
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][nt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun[nt], mx);
      const float alpha = __builtin_amdgcn_exp2f((mrun[nt] - mnew) * cs);
      const float moff = -mnew * cs;
      mrun[nt] = mnew;
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[t][nt][r], cs, moff));
          sacc[t][nt][r] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32);
      lrun[nt] = lrun[nt] * alpha + rs;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
    }

    // ---- O^T += V^T P^T ----------------------------------------------------------------
#pragma unroll
    for (int t = 0; t < C::KT; ++t) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int pc = 2 * t + u;
        bf16x8 pb[C::NT];
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt) {
          uint4 w;
          w.x = pack_bf16x2(sacc[t][nt][8 * u + 0], sacc[t][nt][8 * u + 1]);
          w.y = pack_bf16x2(sacc[t][nt][8 * u + 2], sacc[t][nt][8 * u + 3]);
          w.z = pack_bf16x2(sacc[t][nt][8 * u + 4], sacc[t][nt][8 * u + 5]);
          w.w = pack_bf16x2(sacc[t][nt][8 * u + 6], sacc[t][nt][8 * u + 7]);
          pb[nt] = __builtin_bit_cast(bf16x8, w);
        }
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt) {
          const bf16x8 va = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const uint4*>(ldsV + (32 * dt + l32) * C::VROW + (16 * pc + 8 * hf) * 2));
#pragma unroll
          for (int nt = 0; nt < C::NT; ++nt)
            oacc[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[nt], oacc[dt][nt], 0, 0, 0);
        }
      }
    }
  }

  // ---- epilogue: normalise, rectify, compensate, store ------------------------------------
  __syncthreads();   // comp[] is complete (and nobody still reads the tiles)
  const float rfac = (sparse_row && (a.flags & RSA_RECTIFY_CRITICAL)) ? a.R[vrow] : 1.0f;
  uint16_t* Ob = a.O + base;
#pragma unroll
  for (int nt = 0; nt < C::NT; ++nt) {
    const int q = wave * QW + 32 * nt + l32;
    if (q >= q_count) continue;
    const float f = rfac / lrun[nt];
    uint16_t* orow = Ob + (q_t0 + q) * dm.st;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d0 = 32 * dt + 8 * g + 4 * hf;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = oacc[dt][nt][4 * g + e] * f;
          if (do_comp) o[e] += comp[0][d0 + e] + comp[1][d0 + e];
        }
        uint2 w;
        w.x = pack_bf16x2(o[0], o[1]);
        w.y = pack_bf16x2(o[2], o[3]);
        *reinterpret_cast<uint2*>(orow + d0) = w;
      }
    if (a.lse && hf == 0)
      a.lse[((size_t)bh * dm.t) + q_t0 + q] = mrun[nt] * dm.scale + logf(lrun[nt]);
  }
}

template <int D, int BLK, int QW>
hipError_t launch_attn_t(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  using C = AttnCfg<D, BLK, QW>;
  const int bh = dm.batch * dm.heads;
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int n_text_items = dense_all ? bh * dm.m : bh * dm.mt;
  const int chunk = (dm.n + 7) / 8;
  const long long grid = (long long)n_text_items + (dense_all ? 0 : (long long)bh * 8 * chunk);
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_kernel<D, BLK, QW>), dim3((unsigned)grid), dim3(C::NTHR), 0, s, dm, a, n_text_items, chunk);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_attn_t<128, 128, 32>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_attn_t<128, 64, 32>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_attn_t<64, 128, 32>(dm, a, s);
  return launch_attn_t<64, 64, 32>(dm, a, s);
}

}  // namespace rsa
