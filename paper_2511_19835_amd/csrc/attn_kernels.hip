// Block-sparse flash attention with the rectification fused into the epilogue
// (paper Sec. 3.1 sparse attention, Alg. 1 steps 16-17; Sec. 4.1 / 4.2, Alg. 1 steps 19-23).
//
// A workgroup is eight waves and owns 256 query rows of one (batch, head): groups of BLK/32 waves,
// one group per query block (two at BLK = 128, four at BLK = 64), one wave per 32 query rows,
// groups g and g + NGRP/2 on the same SIMDs. Video query blocks walk their
// compact, ascending list of critical key blocks; text query blocks (and every block under
// RSA_DENSE) walk all M key blocks. Key blocks are consumed in steps of KVS keys. For each
// step the K rows [KVS][d] and the channel-major V rows [d][KVS] of a group are brought into
// its own two-stage LDS ring by direct-to-LDS loads (global_load_lds_dwordx4: no staging
// registers), one step ahead. Each wave computes, with v_mfma_f32_32x32x16_bf16,
//     S^T = K Q^T      (M = key, N = query, k = channel)      -> accumulators: one query
//     O^T += V^T P^T   (M = channel, N = query, k = key)         column per lane
// so the online softmax is lane-local except for one exchange between the two half-waves,
// and the probabilities a lane holds after the first product are exactly the B operand it
// needs for the second (rsa_pool stores V in that key order).
//
// A step of a group is two phases, separated by workgroup barriers: an MFMA phase (the P V
// product of the previous step, then K Q^T of this one: nothing but matrix instructions, LDS
// operand reads a fixed number of slots ahead and the requests for the next tile, one per
// slot) and a softmax phase (VALU only; it also moves the step's V^T operands to registers).
// The two groups run one barrier apart, so that on every SIMD one wave feeds the matrix pipe
// while the other uses the VALU. Measured against one workgroup per query block with the
// softmax interleaved into each wave's own MFMA stream (two workgroups per CU): 14 % fewer
// core cycles, 8 % less time (the clock drops further under the power cap).
// Epilogue: O = R_n * acc / l + C_n, C_n = sum_{m: not kept and M_c} A^pool[n][m] v^pool_m
// (computed beforehand by compensation_kernel into the workspace).
//
// 4*B*B*d flop per (query block, key block) pair against 2*B*d*2 bytes of K/V traffic.
// Workgroups are ordered so that the long dense text rows start first and each XCD
// (workgroup id modulo 8) owns a contiguous range of launch positions of a head;
// row_order_kernel maps positions to video query blocks so that blocks with similar lists
// are resident together (the two of a workgroup are neighbours in that order) and share
// K/V tiles in the XCD's L2.
#include "rsa_common.hpp"
#include "lds_dma.hpp"

namespace rsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#ifndef RSA_KVS
#define RSA_KVS 64
#endif
#ifndef RSA_NSTAGE
#define RSA_NSTAGE 2
#endif
constexpr int KSTAGES = RSA_NSTAGE;  // LDS ring depth of the K tiles of a group
constexpr int VSTAGES = 3;           // ... of its V^T tiles, which are read one phase later than the K tile of the same step
#ifndef RSA_MWIN
#define RSA_MWIN 4
#endif
#ifndef RSA_DSLOT
#define RSA_DSLOT 2
#endif
#ifndef RSA_LSTRIDE
#define RSA_LSTRIDE 1
#endif
constexpr int MWIN = RSA_MWIN;      // MFMA slots between the LDS read of a K operand and its use

template <int D, int BLK>
struct AttnCfg {
  static constexpr int NW = BLK / 32;       // waves per group (one per 32 query rows)
  static constexpr int NGRP = 8 / NW;       // groups = query blocks per workgroup: eight waves, two per SIMD
  static constexpr int NTHR = 64 * NW * NGRP;
  // keys per step; halved where four rings of 64 keys x 128 channels would not fit the LDS
  static constexpr int KVS = (BLK == 64 && D == 128) ? RSA_KVS / 2 : RSA_KVS;
  static constexpr int SPB = BLK / KVS;     // steps per key block
  static constexpr int KT = KVS / 32;       // key tiles of S^T per step
  static constexpr int KS = D / 16;         // k-steps of K Q^T
  static constexpr int DT = D / 32;         // channel tiles of O^T
  static constexpr int PC = KVS / 16;       // 16-key chunks per step
  static constexpr int KCPR = D / 8;        // 16-byte chunks per K row
  static constexpr int VCPR = KVS / 8;      // 16-byte chunks per V^T row of one step
  static constexpr int KINST = KVS * KCPR / 64;   // 1 KB direct-to-LDS loads per K step tile
  static constexpr int VINST = D * VCPR / 64;     // ... per V^T step tile
  static constexpr int KPW = KINST / NW;    // per wave
  static constexpr int VPW = VINST / NW;
  static constexpr int KBUF = KVS * KCPR;   // 16-byte chunks per K buffer
  static constexpr int VBUF = D * VCPR;     // ... per V^T buffer
  static constexpr int GROUP = KSTAGES * KBUF + VSTAGES * VBUF;   // 16-byte chunks of one group: [K stages | V^T stages]
  static_assert(KINST % NW == 0 && VINST % NW == 0, "loads must split evenly over the waves");
  static_assert(KSTAGES == 2 && NGRP * GROUP * 16 <= 160 * 1024, "the rings of all groups must fit the LDS of a CU");
  static_assert(SPB == 1 || SPB == 2, "the main loop is unrolled twice: over the K stages and over the steps of a key block");
  static_assert(NGRP % 2 == 0 && BLK % KVS == 0, "groups pair up on the SIMDs; a block is a whole number of steps");
};

// LDS tiles are unpadded; the 16-byte chunk c of row r is stored at chunk position
// c ^ key(r) so that 16 consecutive rows read at one logical chunk index hit 16 different
// positions (all banks once). CPR = chunks per row (8 or 16).
template <int CPR>
__device__ __forceinline__ int swz_key(int r) { return (r / (16 / CPR)) & (CPR - 1); }
template <int CPR>
__device__ __forceinline__ int swizzled(int r, int c) { return r * CPR + (c ^ swz_key<CPR>(r)); }

// Exchange between the two half-waves (lane l <-> lane l^32) with v_permlane32_swap.
// The vector elements are copied to scalars before the bit casts: a bit cast applied
// directly to an element expression reads element 0 whatever the index.
__device__ __forceinline__ void half_wave_pair(float v, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);   // value held by lane l%32
  hi = __builtin_bit_cast(float, r1);   // value held by lane l%32 + 32
}
__device__ __forceinline__ float half_wave_max(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float half_wave_sum(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return lo + hi;
}

// The running softmax reference is only raised when a row's new maximum exceeds it by
// more than this many binades; probabilities then stay below 2^kLazyBits, which fp32 sums
// and bf16 operands hold without loss, and the accumulators are rescaled rarely.
constexpr float kLazyBits = 6.0f;

template <int V>
struct IntC { static constexpr int value = V; };

template <int D, int BLK>
__global__ __launch_bounds__(512, 1) void attn_kernel(Dims dm, AttnArgs a, int n_text_items,
                                                                                  int chunk) {
  using C = AttnCfg<D, BLK>;
  constexpr int KBUF = C::KBUF;
  constexpr int KVS = C::KVS, NGRP = C::NGRP;
  __shared__ u32x4 lds_all[NGRP * C::GROUP];   // per group: KSTAGES K tiles [KVS][d], then VSTAGES V^T tiles [d][KVS]

  // ---- which (batch*head, query block) is this workgroup ---------------------------------
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int tid = threadIdx.x;
  const int wave_wg = __builtin_amdgcn_readfirstlane(tid / 64);
  const int grp = wave_wg / C::NW;                   // which of the query blocks of this workgroup
  const int wave = wave_wg % C::NW;                  // wave inside the group (groups g and g + NGRP/2 share their SIMDs)
  u32x4* lds = lds_all + grp * C::GROUP;
  int bh;
  int qb_of[NGRP];                                   // query block of every group, -1: none
  {
    const int id = blockIdx.x;
    if (id < n_text_items) {           // long dense rows first, two per workgroup
      const int per = dense_all ? dm.m : dm.mt, pairs = (per + NGRP - 1) / NGRP;
      bh = id / pairs;
      const int r0 = NGRP * (id % pairs), first = dense_all ? 0 : dm.n;
#pragma unroll
      for (int g = 0; g < NGRP; ++g) qb_of[g] = r0 + g < per ? first + r0 + g : -1;
    } else {
      const int v = id - n_text_items;
      const int xcd = v & 7, j = v >> 3, pairs = (chunk + NGRP - 1) / NGRP;
      bh = j / pairs;
      const int p0 = xcd * chunk + NGRP * (j % pairs);              // launch positions p0 .. p0 + NGRP - 1
      const int pend = min(dm.n, (xcd + 1) * chunk);
      if (p0 >= pend) return;          // whole workgroup leaves before any barrier
#pragma unroll
      for (int g = 0; g < NGRP; ++g) {
        qb_of[g] = -1;
        if (p0 + g < pend) qb_of[g] = a.row_order ? a.row_order[(size_t)bh * dm.n + p0 + g] : p0 + g;
      }
    }
  }
  auto steps_of = [&](int qbx) __attribute__((always_inline)) {
    if (qbx < 0) return 0;
    const bool sp = !dense_all && qbx < dm.n;
    return (sp ? a.count[(size_t)bh * dm.n + qbx] : dm.m) * C::SPB;
  };
  int smax = 0;                                      // every group turns the loop this often
#pragma unroll
  for (int g = 0; g < NGRP; ++g) smax = max(smax, steps_of(qb_of[g]));
  const int qb = qb_of[grp] < 0 ? 0 : qb_of[grp];
  const bool active = qb_of[grp] >= 0;
  const int b = bh / dm.heads, h = bh % dm.heads;
  const bool sparse_row = !dense_all && qb < dm.n;
  const size_t vrow = (size_t)bh * dm.n + qb;      // row of the per-video-block tensors
  const int nlist = !active ? 0 : sparse_row ? a.count[vrow] : dm.m;
  const int32_t* list = sparse_row ? a.block_idx + vrow * dm.m : nullptr;

  const int lane = tid % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int64_t base = (int64_t)b * dm.sb + (int64_t)h * dm.sh;
  const uint16_t* Qb = a.Q + base;
  const uint16_t* Kb = a.K + base;
  const uint16_t* Vtb = a.Vt + (size_t)bh * dm.m * D * BLK;

  // ---- direct-to-LDS loads ---------------------------------------------------------------
  // A load fills 1 KB of LDS = RK consecutive K rows (RV consecutive V^T rows). Load ii of
  // wave w covers rows pass*ROWS_PER_PASS + (class*NW + w)*RK + (lane / chunks-per-row): the
  // swizzle key of a lane's row then depends on the class only, so KOFF (usually 1) per-lane
  // byte offsets serve all of a wave's loads and everything else is scalar.
  constexpr int RK = 64 / C::KCPR, RV = 64 / C::VCPR;
  constexpr int KOFF = (C::NW * RK >= 16) ? 1 : 16 / (C::NW * RK);
  constexpr int VOFF = (C::NW * RV >= 16) ? 1 : 16 / (C::NW * RV);
  static_assert(C::KPW % KOFF == 0 && C::VPW % VOFF == 0, "row classes must divide a wave's loads");
  int k_r0[KOFF], k_col[KOFF];
  uint32_t k_voff[KOFF], v_voff[VOFF];
#pragma unroll
  for (int c = 0; c < KOFF; ++c) {
    k_r0[c] = (c * C::NW + wave) * RK + lane / C::KCPR;
    k_col[c] = ((lane % C::KCPR) ^ swz_key<C::KCPR>(k_r0[c])) * 8;              // element offset in the row
    k_voff[c] = (uint32_t)((k_r0[c] * dm.st + k_col[c]) * 2);
  }
#pragma unroll
  for (int c = 0; c < VOFF; ++c) {
    const int r0 = (c * C::NW + wave) * RV + lane / C::VCPR;
    v_voff[c] = (uint32_t)((r0 * BLK + ((lane % C::VCPR) ^ swz_key<C::VCPR>(r0)) * 8) * 2);
  }
  constexpr int K_ROWS_PER_PASS = C::NW * RK * KOFF, V_ROWS_PER_PASS = C::NW * RV * VOFF;
  constexpr int K_LDS_CLASS = C::NW * RK * C::KCPR * 16, V_LDS_CLASS = C::NW * RV * C::VCPR * 16;
  constexpr int K_LDS_PASS = K_ROWS_PER_PASS * C::KCPR * 16, V_LDS_PASS = V_ROWS_PER_PASS * C::VCPR * 16;
  const uint32_t ldsK_addr = (uint32_t)(uintptr_t)lds + wave * RK * (C::KCPR * 16);
  const uint32_t ldsV_addr = (uint32_t)(uintptr_t)lds + KSTAGES * KBUF * 16 + wave * RV * (C::VCPR * 16);

  const int nsteps = nlist * C::SPB;
  // The list is read through the constant address space: a scalar load, which neither waits
  // for nor is held up by the direct-to-LDS loads in flight (a vector load would be both).
  // A dense row has no list (with RSA_DENSE every list pointer may be NULL): its loads read the first
  // word of Q instead, and the index itself is taken.
  typedef const int32_t __attribute__((address_space(4))) * const_list_t;
  const const_list_t clist = (const_list_t)(uintptr_t)(list ? (const void*)list : (const void*)Qb);   // Q: never NULL, at least one row long
  const bool has_list = list != nullptr;
  // entry j of the list; past its end the last entry again (a valid block: the tile requested for a
  // step that does not exist is never read)
  auto list_entry = [&](int j) __attribute__((always_inline)) {
    j = min(j, nlist - 1);
    const int e = clist[has_list ? j : 0];
    return has_list ? e : j;
  };
  // Requests for the K rows and the V^T rows of one step. Everything that does not depend on the
  // step is worked out once, in bytes: load ii of a wave is a per-lane byte offset (kvo / vvo, the
  // pass folded in) from the tile's scalar base and a constant LDS offset from the stage's scalar
  // base, so that a request is one scalar add into M0 and the load itself, and a tile is prepared
  // from its block index with a dozen scalar instructions.
  const uint32_t kblock_bytes = (uint32_t)BLK * (uint32_t)dm.st * 2u;       // K rows of consecutive key blocks
  const uint32_t kstep_bytes = (uint32_t)KVS * (uint32_t)dm.st * 2u;        // ... of consecutive steps inside a block
  const uint32_t kpass_bytes = (uint32_t)K_ROWS_PER_PASS * (uint32_t)dm.st * 2u;
  const int64_t text_adjust = ((int64_t)dm.tv - (int64_t)dm.n * BLK) * dm.st * 2;   // text blocks start at T_v, not N*B
  const int last_video_count = dm.block_count(dm.n - 1), last_count = dm.block_count(dm.m - 1);
  const uint64_t Kbytes = (uint64_t)(uintptr_t)Kb;
  const uint64_t Vtbytes = (uint64_t)(uintptr_t)Vtb;
  constexpr uint32_t kVtBlockBytes = (uint32_t)D * BLK * 2u;
  auto count_of = [&](int m) __attribute__((always_inline)) {
    int c = BLK;
    if (m == dm.n - 1) c = last_video_count;
    if (m == dm.m - 1) c = last_count;
    return c;
  };
  constexpr int LPS = C::KPW + C::VPW;           // loads per step per wave
  uint32_t kvo[C::KPW], vvo[C::VPW];             // per-lane byte offsets of this wave's loads of a full tile
#pragma unroll
  for (int ii = 0; ii < C::KPW; ++ii) kvo[ii] = k_voff[ii % KOFF] + (uint32_t)(ii / KOFF) * kpass_bytes;
#pragma unroll
  for (int ii = 0; ii < C::VPW; ++ii) vvo[ii] = v_voff[ii % VOFF] + (uint32_t)((ii / VOFF) * (V_ROWS_PER_PASS * BLK * 2));
  uint32_t kvw[C::KPW];                          // the K offsets in use: kvo, or clamped rows for a ragged block
#pragma unroll
  for (int ii = 0; ii < C::KPW; ++ii) kvw[ii] = kvo[ii];
  int kvw_ragged = 0;
  struct Tile {
    uint64_t kp;          // K rows of this step (of the whole block when it is ragged)
    uint64_t vp;          // V^T rows of this step
    uint32_t kdst, vdst;  // LDS byte addresses of this wave's first load into the stage
  };
  // The key block whose tiles are being requested: start of its K rows and V^T rows, valid keys.
  uint64_t blk_kp = 0, blk_vp = 0;
  int blk_count = BLK;
  // A tile is prepared in short pieces of scalar work so that the caller can put one behind each
  // of its first MFMAs: open_block for the first step of a key block, step_of_block for every step.
  // A ragged key block (the last video block, the last text block) adds vector work: K rows past
  // the block end re-read its last row (masked later; V^T is zero-padded in HBM), with per-lane
  // offsets from the start of the block.
  auto open_block = [&](int m) __attribute__((always_inline)) {
    blk_kp = Kbytes + ((uint64_t)(uint32_t)m * kblock_bytes + (uint64_t)(m >= dm.n ? text_adjust : 0));
    blk_vp = Vtbytes + (uint64_t)(uint32_t)m * kVtBlockBytes;
    blk_count = count_of(m);
  };
  auto step_of_block = [&](Tile& t, uint32_t part, int kst, int vst) __attribute__((always_inline)) {
    t.kp = blk_kp + part * kstep_bytes;
    t.vp = blk_vp + part * (KVS * 2u);
    t.kdst = ldsK_addr + kst * (KBUF * 16);
    t.vdst = ldsV_addr + vst * (C::VBUF * 16);
    if (kvw_ragged) {
#pragma unroll
      for (int ii = 0; ii < C::KPW; ++ii) kvw[ii] = kvo[ii];
      kvw_ragged = 0;
    }
    if (blk_count < BLK) {
      t.kp = blk_kp;
#pragma unroll
      for (int ii = 0; ii < C::KPW; ++ii) {
        int r = (int)part * KVS + (ii / KOFF) * K_ROWS_PER_PASS + k_r0[ii % KOFF];
        r = r < blk_count ? r : blk_count - 1;
        kvw[ii] = (uint32_t)((r * dm.st + k_col[ii % KOFF]) * 2);
      }
      kvw_ragged = 1;
    }
  };
  auto issue_load = [&](const Tile& t, int idx) __attribute__((always_inline)) {
    if (idx < C::KPW) {
      const int ii = idx;
      dma16_sv_at(t.kdst, (ii / KOFF) * K_LDS_PASS + (ii % KOFF) * K_LDS_CLASS, t.kp, kvw[ii], lds);
    } else {
      const int ii = idx - C::KPW;
      dma16_sv_at(t.vdst, (ii / VOFF) * V_LDS_PASS + (ii % VOFF) * V_LDS_CLASS, t.vp, vvo[ii], lds);
    }
  };

  // ---- loop-invariant LDS read positions (16-byte chunk index inside stage 0, tile 0) ----
  const u32x4* kread[C::KS];
  const u32x4* vread[C::PC];
#pragma unroll
  for (int ks = 0; ks < C::KS; ++ks) kread[ks] = lds + swizzled<C::KCPR>(l32, 2 * ks + hf);
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) vread[pc] = lds + KSTAGES * KBUF + swizzled<C::VCPR>(l32, 2 * pc + hf);

  // ---- Q as the B operand of S^T = K Q^T, resident in registers --------------------------
  const int q_count = dm.block_count(qb);
  const int64_t q_t0 = dm.block_start(qb);
  bf16x8 qreg[C::KS];
  {
    const int q = wave * 32 + l32;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (q < q_count) v = *reinterpret_cast<const uint4*>(Qb + (q_t0 + q) * dm.st + 16 * s + 8 * hf);
      qreg[s] = __builtin_bit_cast(bf16x8, v);
    }
    // Q must have arrived before the first direct-to-LDS load is requested: the compiler
    // does not see those loads, and would otherwise place its own wait for Q -- a wait for
    // *every* outstanding load -- at the first use inside the loop.
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }

  floatx16 oacc[C::DT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float mref = -INFINITY, lpart = 0.f;   // softmax reference (log2 domain) and this lane's partial row sum
  const float cs = dm.scale * kLog2e;

  // Two groups of waves share every SIMD (wave w of group 0 and wave w of group 1). They run
  // the same sequence  [M(s) | barrier | V(s) | barrier] ...  one barrier apart, so that while
  // one group issues MFMAs the other does its softmax on the VALU:
  //   M(s): O^T += V^T P^T of step s-1, then S^T = K Q^T of step s: matrix instructions only, the A
  //         operand of each read from LDS a fixed number of slots ahead (V^T tile of step s-1 from
  //         its ring stage (s-1) % 3, K tile of step s from stage s % 2); the loads of tile s+1
  //         (K into stage (s+1) % 2, V^T into stage (s+1) % 3) go out one per MFMA slot
  //   V(s): mask, online softmax -> P as bf16 B operands (VALU only); fetch the list entry of step
  //         s+2; wait for tile s+1; read the first V^T operands of M(s+1) ahead of the barrier
  // The barrier after V(s) publishes tile s+1 to the group. A K stage is rewritten two steps
  // after it was read, a V^T stage (read in M(s+1), one phase after its K tile) three steps after
  // it was filled: by then every wave of the group has passed the barrier that follows its last
  // read.
  int m_nxt = 0;          // key block of the step after the current one
  int kvc_cur = BLK;      // valid keys in the block of the current step
  int kvc_nxt = BLK;
  auto group_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  floatx16 sacc[C::KT];
  u32x4 pb[C::PC];            // probabilities as bf16 B operands, 16 keys per entry
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) pb[pc] = u32x4{0u, 0u, 0u, 0u};

  // M(s) is one fixed sequence of NPV + NQK MFMA slots: the P V product of step s-1, then K Q^T
  // of step s. The A operand of a slot (16 bytes per lane of the V^T or K tile) is read from LDS W
  // slots ahead of its MFMA into a ring of W registers, so that LDS latency stays behind MFMAs
  // that already have their operands; the first W operands of a phase are read at the end of the
  // softmax phase before it. The order is pinned slot by slot.
  constexpr int NPV = C::PC * C::DT, NQK = C::KS * C::KT, NSLOT = NPV + NQK;
  constexpr int W = MWIN;
  static_assert(W - W / 2 <= 4, "the operand waits are written out for at most four reads left outstanding");
  static_assert(NPV >= W && NQK >= W, "the operands read ahead of a phase all belong to its first product");
  bf16x8 ring[W];
#pragma unroll
  for (int i = 0; i < W; ++i) ring[i] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
  int vst = 0;                // V^T ring stage of the current step (s % VSTAGES)
  const u32x4* vcur[C::PC];   // vread[] moved to the V^T stage whose P V product comes next
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) vcur[pc] = vread[pc];
  auto read_v_operand = [&](int slot) __attribute__((always_inline)) {      // slot < NPV
    const int pc = slot / C::DT, dt = slot % C::DT;
    ring[slot % W] = __builtin_bit_cast(bf16x8, vcur[pc][dt * 32 * C::VCPR]);
  };

  auto m_phase = [&](auto stc, auto pvc, auto qkc, int s) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;          // s modulo the unroll factor: gives the K stage and the part of the key block
    constexpr bool do_pv = decltype(pvc)::value != 0, do_qk = decltype(qkc)::value != 0;
    constexpr int DSLOT = RSA_DSLOT;                  // the slot in which the requests for the next tile start
    constexpr int LSTRIDE = RSA_LSTRIDE;              // ... and the slots from one request to the next
    constexpr int FIRST = do_pv ? 0 : NPV, LAST = do_qk ? NSLOT : NPV;     // slots that hold an MFMA
    constexpr int WB = W / 2;                         // operands are waited for WB at a time
    Tile nt = {};
    auto read_k_operand = [&](int slot) __attribute__((always_inline)) {   // slot >= NPV
      const int q = slot - NPV, k2 = q / C::KT, t = q % C::KT;
      ring[slot % W] = __builtin_bit_cast(bf16x8, kread[k2][(ST % KSTAGES) * KBUF + t * 32 * C::KCPR]);
    };
    auto read_operand = [&](int slot) __attribute__((always_inline)) {
      if (slot < NPV) read_v_operand(slot); else read_k_operand(slot);
    };
    // The wave that feeds the matrix pipe goes first wherever the two waves of a SIMD compete for an
    // issue slot: without this the older wave of the two wins, and the MFMA phases of the younger
    // group run a fifth longer than those of the other.
    __builtin_amdgcn_s_setprio(3);
    if (!do_pv) {
      // first step of a list: nothing was read ahead
#pragma unroll
      for (int j = FIRST; j < FIRST + W && j < LAST; ++j) read_operand(j);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = FIRST; i < LAST; ++i) {
      const int e = i - FIRST;                        // position among the MFMAs of this phase
      // The operands of slots i .. i+WB-1 have arrived once at most the reads behind them are
      // outstanding: one wait per WB slots, and none is needed in between.
      if (e % WB == 0) {
        const int behind = min(W - WB, max(LAST - i - WB, 0));
        // vmcnt and expcnt fields at "no wait", lgkmcnt = behind
        if (behind == 0) __builtin_amdgcn_s_waitcnt(0xC07F);
        else if (behind == 1) __builtin_amdgcn_s_waitcnt(0xC17F);
        else if (behind == 2) __builtin_amdgcn_s_waitcnt(0xC27F);
        else if (behind == 3) __builtin_amdgcn_s_waitcnt(0xC37F);
        else __builtin_amdgcn_s_waitcnt(0xC47F);
        __builtin_amdgcn_sched_barrier(0);
      }
      // one load of the tile of step s+1 per slot, behind the MFMA of the slot before
      if (do_qk && e >= DSLOT && (e - DSLOT) % LSTRIDE == 0 && (e - DSLOT) / LSTRIDE < LPS) issue_load(nt, (e - DSLOT) / LSTRIDE);
      if (i < NPV) {
        const int pc = i / C::DT, dt = i % C::DT;
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % W], __builtin_bit_cast(bf16x8, pb[pc]), oacc[dt], 0, 0, 0);
      } else {
        const int q = i - NPV, k2 = q / C::KT, t = q % C::KT;
        floatx16 c0 = sacc[t];
        if (k2 == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) c0[r] = 0.f;           // folds into the instruction's constant C operand
        }
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % W], qreg[k2], c0, 0, 0, 0);
      }
      // the ring entry this slot used takes the operand of slot i + W
      if (i + W < LAST) read_operand(i + W);
      if (do_qk && e < 2) {
        // behind the first MFMAs, so that the matrix pipe starts as soon as the barrier opens:
        // addresses of the tile of step s+1. The loop is unrolled over the steps of a key block, so
        // whether that step opens a new block (its list entry came in during V(s-1)) is known at
        // compile time. A list that ends with this step requests the tile of its last entry once
        // more, into a stage nobody reads again.
        __builtin_amdgcn_sched_barrier(0);
        constexpr int PART_NEXT = (ST + 1) % C::SPB;
        if (e == 0) {
          if (PART_NEXT == 0) open_block(m_nxt);
          kvc_nxt = blk_count;
        } else {
          step_of_block(nt, PART_NEXT, (ST + 1) % KSTAGES, vst + 1 >= VSTAGES ? 0 : vst + 1);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // a phase with fewer slots than loads (the first step of a list has no P V product) sends the rest here
#pragma unroll
    for (int idx = 0; idx < LPS; ++idx) {
      if (do_qk && DSLOT + idx * LSTRIDE >= LAST - FIRST) issue_load(nt, idx);
    }
  };

  auto v_phase = [&](auto stc, int s) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;
    __builtin_amdgcn_s_setprio(0);
    {
      const int kv_count = kvc_cur;
      // accumulator register r of key tile t is key part*KVS + 32t + 8(r/4) + 4*hf + r%4 of the block
      if (kv_count < BLK) {
        constexpr int part = ST % C::SPB;
#pragma unroll
        for (int t = 0; t < C::KT; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = part * KVS + 32 * t + 8 * (r / 4) + 4 * hf + (r % 4);
            if (kv >= kv_count) sacc[t][r] = -INFINITY;
          }
      }
      // ---- online softmax, one query column per lane ---------------------------------
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][r]);
      mx = half_wave_max(mx) * cs;
      if (__any(mx > mref + kLazyBits)) {
        const float mnew = fmaxf(mref, mx);
        const float alpha = __builtin_amdgcn_exp2f(mref - mnew);
        mref = mnew;
        lpart *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
      }
      const float moff = -mref;   // finite: the first step of a list always holds a valid key
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < C::KT; ++t) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[t][r], cs, moff));
          rs += p[r];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          u32x4 w;
          w.x = pack_bf16x2(p[8 * u + 0], p[8 * u + 1]);
          w.y = pack_bf16x2(p[8 * u + 2], p[8 * u + 3]);
          w.z = pack_bf16x2(p[8 * u + 4], p[8 * u + 5]);
          w.w = pack_bf16x2(p[8 * u + 6], p[8 * u + 7]);
          pb[2 * t + u] = w;
        }
      }
      lpart += rs;
    }
    // the list entry of step s+2 (where that step opens a key block) for M(s+1), fetched a phase ahead
    if ((ST + 2) % C::SPB == 0) m_nxt = list_entry((s + 2) / C::SPB);
    kvc_cur = kvc_nxt;
    // the probabilities are complete here: nothing of the softmax may sink behind the barrier
    // into the MFMA phase, where it would take the other group's VALU time
#pragma unroll
    for (int pc = 0; pc < C::PC; ++pc) asm volatile("" : "+v"(pb[pc]));
    asm volatile("" : "+v"(lpart), "+v"(mref));
    // the first V^T operands of M(s+1), from the stage of this step (published a whole step ago)
#pragma unroll
    for (int pc = 0; pc < C::PC; ++pc) vcur[pc] = vread[pc] + vst * C::VBUF;
#pragma unroll
    for (int j = 0; j < W; ++j) read_v_operand(j);
    vst = vst + 1 >= VSTAGES ? 0 : vst + 1;
    // tile s+1 has landed (this wave's share; the barrier that follows covers the group)
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  };

  if (nsteps > 0) {
    Tile t0;
    open_block(list_entry(0));
    step_of_block(t0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < LPS; ++i) issue_load(t0, i);
    kvc_cur = blk_count;
    if (C::SPB == 1) m_nxt = list_entry(1);       // otherwise V(0) fetches it
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  group_barrier();                  // tile 0 of both groups is in LDS
  if (grp >= NGRP / 2) group_barrier();    // the second half of the groups runs one barrier behind the first
  // Every group turns smax + 1 rounds of two barriers; a round is M(s), V(s) while the group has
  // steps left, the last P V product alone in round nsteps, and nothing but the barriers after.
  using Y = IntC<1>;
  using N = IntC<0>;
  int s = 0;
  if (nsteps > 0) {
    m_phase(IntC<0>{}, N{}, Y{}, 0);
    group_barrier();
    v_phase(IntC<0>{}, 0);
    group_barrier();
    s = 1;
    while (s + 1 < nsteps) {        // s is odd here
      m_phase(IntC<1>{}, Y{}, Y{}, s);
      group_barrier();
      v_phase(IntC<1>{}, s);
      group_barrier();
      m_phase(IntC<0>{}, Y{}, Y{}, s + 1);
      group_barrier();
      v_phase(IntC<0>{}, s + 1);
      group_barrier();
      s += 2;
    }
    if (s < nsteps) {
      m_phase(IntC<1>{}, Y{}, Y{}, s);
      group_barrier();
      v_phase(IntC<1>{}, s);
      group_barrier();
      s += 1;
    }
    if (s & 1) m_phase(IntC<1>{}, Y{}, N{}, s); else m_phase(IntC<0>{}, Y{}, N{}, s);
    group_barrier();
    group_barrier();
    s += 1;
  }
  for (; s <= smax; ++s) {
    group_barrier();
    group_barrier();
  }
  if (grp < NGRP / 2) group_barrier();

  if (!active) return;      // no barrier follows

  // ---- epilogue: normalise, rectify, compensate, store ------------------------------------
  const bool do_comp = sparse_row && (a.flags & RSA_COMPENSATE);
  const float rfac = (sparse_row && (a.flags & RSA_RECTIFY_CRITICAL)) ? a.R[vrow] : 1.0f;
  uint16_t* Ob = a.O + base;
  {
    const float lsum = half_wave_sum(lpart);
    const int q = wave * 32 + l32;
    if (q < q_count) {
      const float f = rfac / lsum;
      uint16_t* orow = Ob + (q_t0 + q) * dm.st;
      const float* crow = a.comp + vrow * D;     // C_n of this query block (only read when do_comp)
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int d0 = 32 * dt + 8 * g + 4 * hf;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = oacc[dt][4 * g + e] * f;
          if (do_comp) {
            const floatx4 c4 = *reinterpret_cast<const floatx4*>(crow + d0);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] += c4[e];
          }
          uint2 w;
          w.x = pack_bf16x2(o[0], o[1]);
          w.y = pack_bf16x2(o[2], o[3]);
          *reinterpret_cast<uint2*>(orow + d0) = w;
        }
      if (a.lse && hf == 0)
        a.lse[((size_t)bh * dm.t) + q_t0 + q] = (mref + log2f(lsum)) * 0.6931471805599453f;
    }
  }
}

// Pooled compensation (Alg. 1 step 21): C[n][:] = sum over blocks m that are not kept and
// have their M_c bit set of A^pool[n][m] * v^pool[m][:], all fp32, blocks in ascending order.
// Most blocks are not compensated (the gate is off, or the block is kept), so the sum runs over
// the set bits only. One wave per query block: lane l looks at block 64 s + l of slot s (its
// bit, its weight: one coalesced read of the row of A^pool), a ballot gives the slot's
// compensated blocks, and for each of them, eight at a time so that their loads are in flight
// together, the weight is broadcast from its lane and the row of v^pool (L2 resident) is added,
// every lane owning D/64 channels. Padding entries of a group of eight carry weight 0 and add
// exactly nothing.
template <int D>
__global__ __launch_bounds__(256) void compensation_kernel(Dims dm, AttnArgs a) {
  constexpr int CPL = D / 64;                    // channels per lane
  constexpr int U = 8;                           // blocks per group
  const int lane = threadIdx.x % 64;
  const int n = blockIdx.x * 4 + (int)(threadIdx.x / 64), bh = blockIdx.y;
  if (n >= dm.n) return;                         // no barriers in this kernel
  const size_t row = (size_t)bh * dm.n + n;
  const uint32_t* kept = a.mask_bits + row * dm.w;
  const uint32_t* gate = a.Mc_bits + row * dm.w;
  const float* A = a.Apool + row * dm.m;
  const float* Vp = a.Vp + (size_t)bh * dm.m * D + lane;
  float acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
  const int slots = (dm.m + 63) / 64;
  // this lane's block of a slot: is it compensated, and its weight (read a slot ahead of its use)
  auto look = [&](int s, bool& on, float& wl) __attribute__((always_inline)) {
    const int m = 64 * s + lane, word = 2 * s + (lane >> 5);
    on = false;
    wl = 0.f;
    if (m < dm.m) {
      on = ((~kept[word] & gate[word]) >> (lane & 31)) & 1u;
      if (on) wl = A[m];
    }
  };
  bool on_next;
  float wl_next;
  look(0, on_next, wl_next);
  for (int s = 0; s < slots; ++s) {
    const bool on = on_next;
    const float wl = wl_next;
    if (s + 1 < slots) look(s + 1, on_next, wl_next);
    unsigned long long todo = __ballot(on);
    while (todo) {
      int src[U];
      float wt[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        src[u] = todo ? __builtin_ctzll(todo) : 0;           // wave-uniform
        wt[u] = todo ? __shfl(wl, src[u]) : 0.f;
        todo &= todo - 1;                                    // 0 stays 0
      }
      float v[U][CPL];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CPL; ++c) v[u][c] = Vp[(size_t)(64 * s + src[u]) * D + 64 * c];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] = fmaf(wt[u], v[u][c], acc[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < CPL; ++c) a.comp[row * D + lane + 64 * c] = acc[c];
}

// Launch order of the video query blocks of one (batch, head): sorted by their first three
// kept key blocks (ties: block index). Workgroups that are resident on an XCD at the same time
// then walk similar lists and find each other's K/V tiles in that XCD's L2 (on the benchmark
// inputs the traffic that crosses the fabric drops by 40 %). A heuristic: any permutation gives
// the same results. One workgroup per (batch, head), bitonic sort of 64-bit keys in LDS.
__global__ __launch_bounds__(1024) void row_order_kernel(Dims dm, AttnArgs a) {
  __shared__ uint64_t keys[RSA_MAX_BLOCKS];
  const int bh = blockIdx.x, tid = threadIdx.x;
  int P = 1;
  while (P < dm.n) P <<= 1;
  for (int i = tid; i < P; i += 1024) {
    uint64_t k = ~0ull;                                    // padding sorts to the end
    if (i < dm.n) {
      const size_t row = (size_t)bh * dm.n + i;
      const int cnt = a.count[row];
      const int32_t* lst = a.block_idx + row * dm.m;
      const uint64_t i0 = cnt > 0 ? lst[0] : 4095, i1 = cnt > 1 ? lst[1] : 4095, i2 = cnt > 2 ? lst[2] : 4095;
      k = (i0 << 36) | (i1 << 24) | (i2 << 12) | (uint64_t)i;     // every index < RSA_MAX_BLOCKS = 2^12
    }
    keys[i] = k;
  }
  __syncthreads();
  for (int k2 = 2; k2 <= P; k2 <<= 1)
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < P; i += 1024) {
        const int o = i ^ j;
        if (o > i) {
          const uint64_t x = keys[i], y = keys[o];
          if ((x > y) == ((i & k2) == 0)) {
            keys[i] = y;
            keys[o] = x;
          }
        }
      }
      __syncthreads();
    }
  for (int i = tid; i < dm.n; i += 1024) a.row_order[(size_t)bh * dm.n + i] = (int32_t)(keys[i] & 4095u);
}

template <int D, int BLK>
hipError_t launch_attn_t(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  using C = AttnCfg<D, BLK>;
  const int bh = dm.batch * dm.heads;
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  constexpr int G = C::NGRP;                                                       // query blocks per workgroup
  const int n_text_items = bh * (((dense_all ? dm.m : dm.mt) + G - 1) / G);       // workgroups of dense rows
  const int chunk = (dm.n + 7) / 8;
  const long long grid = (long long)n_text_items + (dense_all ? 0 : (long long)bh * 8 * ((chunk + G - 1) / G));
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  if (!dense_all && (a.flags & RSA_COMPENSATE))
    hipLaunchKernelGGL((compensation_kernel<D>), dim3((dm.n + 3) / 4, bh), dim3(256), 0, s, dm, a);
  if (!dense_all && a.row_order) hipLaunchKernelGGL(row_order_kernel, dim3(bh), dim3(1024), 0, s, dm, a);
  hipLaunchKernelGGL((attn_kernel<D, BLK>), dim3((unsigned)grid), dim3(C::NTHR), 0, s, dm, a, n_text_items, chunk);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_attn_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_attn_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_attn_t<64, 128>(dm, a, s);
  return launch_attn_t<64, 64>(dm, a, s);
}

}  // namespace rsa
