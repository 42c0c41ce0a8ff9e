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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int D, int BLK, int QW>
struct AttnCfg {
  static constexpr int NW = BLK / QW;       // waves per workgroup
  static constexpr int NTHR = 64 * NW;
  static constexpr int NT = QW / 32;        // query tiles per wave
  static constexpr int KT = BLK / 32;       // key tiles of S^T
  static constexpr int KS = D / 16;         // k-steps of K Q^T
  static constexpr int DT = D / 32;         // channel tiles of O^T
  static constexpr int KCPR = D / 8;        // 16-byte chunks per K row
  static constexpr int VCPR = BLK / 8;      // 16-byte chunks per V^T row
  static constexpr int KLD = BLK * KCPR / NTHR;  // chunks each thread moves per K tile
  static constexpr int VLD = D * VCPR / NTHR;    // ... per V^T tile
  static constexpr int NSTAGE = KLD > VLD ? KLD : VLD;
  static constexpr int MINW = QW == 32 ? 2 : 1;  // waves per SIMD the register budget must allow
};

// LDS tiles are unpadded; the 16-byte chunk c of row r is stored at chunk position
// c ^ key(r) so that 16 consecutive rows read at one logical chunk index hit 16 different
// positions (all banks once). CPR = chunks per row (8 or 16).
template <int CPR>
__device__ inline int swizzled(int r, int c) {
  return r * CPR + (c ^ ((r / (16 / CPR)) & (CPR - 1)));
}

// Exchange between the two half-waves (lane l <-> lane l^32) with v_permlane32_swap.
// The vector elements are copied to scalars before the bit casts: a bit cast applied
// directly to an element expression reads element 0 whatever the index.
__device__ inline void half_wave_pair(float v, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);   // value held by lane l%32
  hi = __builtin_bit_cast(float, r1);   // value held by lane l%32 + 32
}
__device__ inline float half_wave_max(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return fmaxf(lo, hi);
}
__device__ inline float half_wave_sum(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return lo + hi;
}

// Tile movers. A K tile is BLK rows of the caller's K (row stride st); a V^T tile is the
// contiguous D x BLK block rsa_pool wrote. Each thread carries NLD 16-byte chunks.
template <class C>
__device__ __forceinline__ void fetch_k_tile(u32x4 (&stage)[C::NSTAGE], const uint16_t* Kb, const Dims& dm, int m,
                                             int tid) {
  const int kv_count = dm.block_count(m);
  const uint16_t* src = Kb + dm.block_start(m) * dm.st;
#pragma unroll
  for (int i = 0; i < C::KLD; ++i) {
    const int slot = tid + i * C::NTHR;
    int r = slot / C::KCPR;
    const int c = slot % C::KCPR;
    r = r < kv_count ? r : kv_count - 1;   // rows past a ragged block re-read its last row (masked later)
    stage[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)r * dm.st + c * 8);
  }
}
template <class C>
__device__ __forceinline__ void fetch_v_tile(u32x4 (&stage)[C::NSTAGE], const u32x4* src, int tid) {
#pragma unroll
  for (int i = 0; i < C::VLD; ++i) stage[i] = src[tid + i * C::NTHR];
}
template <int NLD, int CPR, int NTHR, int NS>
__device__ __forceinline__ void park_tile(const u32x4 (&stage)[NS], u32x4* lds, int tid) {
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int slot = tid + i * NTHR;
    lds[swizzled<CPR>(slot / CPR, slot % CPR)] = stage[i];
  }
}

// The running softmax reference is only raised when a row's new maximum exceeds it by
// more than this many binades; probabilities then stay below 2^kLazyBits, which fp32 sums
// and bf16 operands hold without loss, and the accumulators are rescaled rarely.
constexpr float kLazyBits = 6.0f;

template <int D, int BLK, int QW>
__global__ __launch_bounds__(64 * BLK / QW, (QW == 32 && BLK == 128 ? 2 : 1)) void attn_kernel(Dims dm, AttnArgs a,
                                                                                int n_text_items, int chunk) {
  using C = AttnCfg<D, BLK, QW>;
  __shared__ u32x4 ldsK[BLK * C::KCPR];
  __shared__ u32x4 ldsV[D * C::VCPR];
  __shared__ float comp[2][D];

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
  float mref[C::NT], lpart[C::NT];   // softmax reference (log2 domain, scaled) and this lane's partial row sum
#pragma unroll
  for (int nt = 0; nt < C::NT; ++nt) { mref[nt] = -INFINITY; lpart[nt] = 0.f; }
  const float cs = dm.scale * kLog2e;

  u32x4 stage[C::NSTAGE];   // one tile in flight: global -> registers -> LDS
  const u32x4* Vt4 = reinterpret_cast<const u32x4*>(Vtb);
#define FETCH_K(m) fetch_k_tile<C>(stage, Kb, dm, (m), tid)
#define PARK_K() park_tile<C::KLD, C::KCPR, C::NTHR>(stage, ldsK, tid)
#define FETCH_V(m) fetch_v_tile<C>(stage, Vt4 + (size_t)(m) * (D * BLK / 8), tid)
#define PARK_V() park_tile<C::VLD, C::VCPR, C::NTHR>(stage, ldsV, tid)

  int m_cur = list ? list[0] : 0;
  if (nlist > 0) {
    FETCH_K(m_cur);
    PARK_K();
    FETCH_V(m_cur);
  }

  for (int j = 0; j < nlist; ++j) {
    const int kv_count = dm.block_count(m_cur);
    const int m_next = (j + 1 < nlist) ? (list ? list[j + 1] : j + 1) : m_cur;
    __syncthreads();   // K tile visible; every wave is past the previous P.V (V tile free)

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
        const bf16x8 ka = __builtin_bit_cast(bf16x8, ldsK[swizzled<C::KCPR>(32 * t + l32, 2 * s + hf)]);
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
    u32x4 pb[C::KT * 2][C::NT];   // probabilities as bf16 B operands, 16 keys per entry
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt) {
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][nt][r]);
      mx = half_wave_max(mx) * cs;
      if (__any(mx > mref[nt] + kLazyBits)) {
        const float mnew = fmaxf(mref[nt], mx);
        const float alpha = __builtin_amdgcn_exp2f(mref[nt] - mnew);
        mref[nt] = mnew;
        lpart[nt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
      }
      const float moff = -mref[nt];
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < C::KT; ++t) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[t][nt][r], cs, moff));
          rs += p[r];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          u32x4 w;
          w.x = pack_bf16x2(p[8 * u + 0], p[8 * u + 1]);
          w.y = pack_bf16x2(p[8 * u + 2], p[8 * u + 3]);
          w.z = pack_bf16x2(p[8 * u + 4], p[8 * u + 5]);
          w.w = pack_bf16x2(p[8 * u + 6], p[8 * u + 7]);
          pb[2 * t + u][nt] = w;
        }
      }
      lpart[nt] += rs;
    }

    PARK_V();                       // V tile of this step: registers -> LDS
    if (j + 1 < nlist) FETCH_K(m_next);
    __syncthreads();                // V tile visible; every wave is past this step's K reads

    // ---- O^T += V^T P^T ----------------------------------------------------------------
#pragma unroll
    for (int pc = 0; pc < C::KT * 2; ++pc) {
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt) {
        const bf16x8 va = __builtin_bit_cast(bf16x8, ldsV[swizzled<C::VCPR>(32 * dt + l32, 2 * pc + hf)]);
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
          oacc[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, pb[pc][nt]),
                                                                 oacc[dt][nt], 0, 0, 0);
      }
    }
    if (j + 1 < nlist) {
      PARK_K();                     // next K tile: registers -> LDS (visible after the barrier that opens the next step)
      FETCH_V(m_next);
    }
    m_cur = m_next;
  }

  // ---- epilogue: normalise, rectify, compensate, store ------------------------------------
  __syncthreads();   // comp[] is complete
  const float rfac = (sparse_row && (a.flags & RSA_RECTIFY_CRITICAL)) ? a.R[vrow] : 1.0f;
  uint16_t* Ob = a.O + base;
#pragma unroll
  for (int nt = 0; nt < C::NT; ++nt) {
    const float lsum = half_wave_sum(lpart[nt]);
    const int q = wave * QW + 32 * nt + l32;
    if (q >= q_count) continue;
    const float f = rfac / lsum;
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
      a.lse[((size_t)bh * dm.t) + q_t0 + q] = (mref[nt] + log2f(lsum)) * 0.6931471805599453f;
  }
#undef FETCH_K
#undef PARK_K
#undef FETCH_V
#undef PARK_V
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
