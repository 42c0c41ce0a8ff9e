// Block-sparse flash attention with the rectification fused into the epilogue
// (paper Sec. 3.1 sparse attention, Alg. 1 steps 16-17; Sec. 4.1 / 4.2, Alg. 1 steps 19-23).
//
// The kernel is persistent: one workgroup of eight waves per CU, in groups of BLK/32 waves (two groups
// at BLK = 128, four at BLK = 64; one wave per 32 query rows; groups g and g + NGRP/2 on the same
// SIMDs). A group works through a sequence of items -- query blocks of some (batch, head) -- that
// schedule_kernel dealt to it, as one unbroken stream of steps: a video query block walks its
// compact, ascending list of critical key blocks, a text query block (and every block under
// RSA_DENSE) all M key blocks, KVS keys per step. For each step the K rows [KVS][d] and the
// channel-major V rows [d][KVS] are brought into the group's own LDS rings by direct-to-LDS loads
// (global_load_lds_dwordx4: no staging registers), one step ahead -- also across the boundary
// between two items, so the matrix pipe never drains. Each wave computes, with
// v_mfma_f32_32x32x16_bf16,
//     S^T = K Q^T      (M = key, N = query, k = channel)      -> accumulators: one query
//     O^T += V^T P^T   (M = channel, N = query, k = key)         column per lane
// so the online softmax is lane-local except for one exchange between the two half-waves,
// and the probabilities a lane holds after the first product are exactly the B operand it
// needs for the second (rsa_pool stores V in that key order).
//
// A step of a group is two phases, separated by workgroup barriers: an MFMA phase (the P V
// product of the previous step, then K Q^T of this one: matrix instructions, their LDS operand
// reads a few slots ahead and the requests for the next tile, one per slot) and a softmax phase
// (VALU only). The groups run one barrier apart, so that on every SIMD one wave feeds the matrix
// pipe while the other uses the VALU. When an item ends its output is written in the softmax phase
// of the next item's first step: O = R_n * acc / l + C_n, C_n = sum_{m: not kept and M_c}
// A^pool[n][m] v^pool_m (computed beforehand by compensation_kernel into the workspace).
//
// 4*B*B*d flop per (query block, key block) pair against 2*B*d*2 bytes of K/V traffic.
// The small kernels named here are in attn_side_kernels.hip. row_order_kernel sorts the video query blocks of a head by their first kept key blocks;
// schedule_kernel deals that order (long dense rows first) to the groups so that each XCD
// (workgroup id modulo 8) owns a contiguous range of it, groups resident together walk similar
// lists and share K/V tiles in the XCD's L2, and all groups end within one item of each other.
#include "attn_sched.hpp"
#include "lds_dma.hpp"
#include "rsa_common.hpp"

namespace rsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
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
constexpr bool SPLIT_LOADS = true;   // K rows requested in the MFMA phase, V^T rows in the softmax phase
constexpr int MWIN = RSA_MWIN;      // MFMA slots between the LDS read of a K operand and its use

template <int D, int BLK>
struct AttnCfg {
  static constexpr int NW = BLK / 32;       // waves per group (one per 32 query rows)
  static constexpr int NGRP = 8 / NW;       // groups = query blocks per workgroup: eight waves, two per SIMD
  static constexpr int NTHR = 64 * NW * NGRP;
  // keys per step: half a key block, so that every key block is two steps and every item an even
  // number of them (the loop over the steps is unrolled twice)
  static constexpr int KVS = BLK / 2;
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
  static_assert(SPB == 2, "the main loop is unrolled twice: over the K stages and over the steps of a key block");
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

// The lane number, worked out where it is asked for. What happens once per item (query rows, epilogue)
// takes its lane-dependent addresses from this: values derived from the lane number at the top of the
// kernel would be live across the whole step loop, where there is no register left for them, and a
// spilled vector register comes back with a wait for every load in flight, tile requests included.
__device__ __forceinline__ int lane_now() {
  int l;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
  return l;
}

// The running softmax reference only moves when a score is more than this many binades away from it
// (above it; in the first step of an item, either way): probabilities then stay within 2^+-kLazyBits of
// one another's scale, far inside what fp32 sums and bf16 operands hold, and the accumulators are
// rescaled very rarely.
constexpr float kLazyBits = 40.0f;

template <int V>
struct IntC { static constexpr int value = V; };
// f(IntC<I>{}) for I = FROM .. TO-1, unrolled at compile time (the index is a constant inside f)
template <int FROM, int TO, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FROM < TO) {
    f(IntC<FROM>{});
    static_for<FROM + 1, TO>(f);
  }
}

// Work of the persistent attention kernel. An item is one query block of one (batch, head); a slot
// is one group of waves of one resident workgroup and works through a sequence of items.
//   table != NULL: schedule_kernel dealt the items to the slots (balanced by their number of steps,
//                  neighbouring rows of the launch order to neighbouring slots at the same time);
//   table == NULL: item i goes to slot i % n_slots (no workspace: index order).
struct SchedArgs {
  const int32_t* table;     // [slots][cap] item records: (batch*heads index) * RSA_MAX_BLOCKS + query block
  const int32_t* nitems;    // [slots]
  const int32_t* total;     // [slots] steps of all items of the slot
  int cap;
  int n_items, n_dense;     // all items; the dense ones (text query blocks, or every block under RSA_DENSE) come first
  int dense_per_bh, dense_first;
};

template <int D, int BLK>
__global__ __launch_bounds__(512, 1) void attn_kernel(Dims dm, AttnArgs a, SchedArgs sc) {
  using C = AttnCfg<D, BLK>;
  constexpr int KBUF = C::KBUF;
  constexpr int KVS = C::KVS, NGRP = C::NGRP;
  __shared__ u32x4 lds_all[NGRP * C::GROUP];   // per group: KSTAGES K tiles [KVS][d], then VSTAGES V^T tiles [d][KVS]

  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int tid = threadIdx.x;
  const int wave_wg = __builtin_amdgcn_readfirstlane(tid / 64);
  const int grp = wave_wg / C::NW;                   // which group of this workgroup
  const int wave = wave_wg % C::NW;                  // wave inside the group (groups g and g + NGRP/2 share their SIMDs)
  const int lane = tid % 64;
  const int l32 = lane % 32, hf = lane / 32;
  u32x4* lds = lds_all + grp * C::GROUP;

  // ---- the items of this group, and how many rounds the workgroup turns -------------------
  // Slots are numbered so that the 64 slots of one schedule queue sit on one XCD (workgroup id
  // modulo 8) and the groups of a workgroup are neighbours in it.
  const int n_wg = gridDim.x, wg = blockIdx.x;
  auto slot_of_group = [&](int g) __attribute__((always_inline)) {
    if (!sc.table) return wg * NGRP + g;
    const int u = (wg / 8) * NGRP + g;
    return ((wg % 8) + 8 * (u / 64)) * 64 + u % 64;
  };
  const int n_slots = n_wg * NGRP;                   // (index-order dealing)
  auto record_of_item = [&](int i) __attribute__((always_inline)) {       // index order: dense items, then video rows
    int bhx, qbx;
    if (i < sc.n_dense) {
      bhx = i / sc.dense_per_bh;
      qbx = sc.dense_first + i % sc.dense_per_bh;
    } else {
      const int v = i - sc.n_dense;
      bhx = v / dm.n;
      qbx = v % dm.n;
    }
    return bhx * RSA_MAX_BLOCKS + qbx;
  };
  auto steps_of_record = [&](int rec) __attribute__((always_inline)) {
    const int bhx = rec / RSA_MAX_BLOCKS, qbx = rec % RSA_MAX_BLOCKS;
    const bool sp = !dense_all && qbx < dm.n;
    return (sp ? list_length(a, dm, (size_t)bhx * dm.n + qbx) : dm.m) * C::SPB;
  };
  const int slot = slot_of_group(grp);
  int n_my_items, wg_rounds = 0;
  if (sc.table) {
    n_my_items = sc.nitems[slot];
#pragma unroll
    for (int g = 0; g < NGRP; ++g) {
      const int t = sc.total[slot_of_group(g)];
      wg_rounds = max(wg_rounds, t > 0 ? t + 1 : 0);
    }
  } else {
    n_my_items = slot < sc.n_items ? (sc.n_items - slot + n_slots - 1) / n_slots : 0;
#pragma unroll
    for (int g = 0; g < NGRP; ++g) {
      int t = 0;
      for (int i = wg * NGRP + g; i < sc.n_items; i += n_slots) t += steps_of_record(record_of_item(i));
      wg_rounds = max(wg_rounds, t > 0 ? t + 1 : 0);
    }
  }
  if (wg_rounds == 0) return;                        // the whole workgroup: nothing was dealt to it
  auto my_record = [&](int k) __attribute__((always_inline)) {
    typedef const int32_t __attribute__((address_space(4))) * const_i32_t;   // scalar loads
    return sc.table ? ((const_i32_t)(uintptr_t)sc.table)[(size_t)slot * sc.cap + k] : record_of_item(slot + k * n_slots);
  };

  // What the phases need to know of an item: all wave-uniform.
  typedef const int32_t __attribute__((address_space(4))) * const_list_t;
  struct Item {
    int bh, qb;
    int ns;                 // steps: SPB per entry of its list (all M key blocks for a dense row)
    int nlist;
    int has_list;
    const_list_t list;      // its list of key blocks; a dense row: any readable address
    uint64_t Kbytes, Vtbytes;   // K rows and V^T tiles of its (batch, head)
    int64_t qo_off;         // element offset of its first query row in Q and in O
    int q_t0, q_count;      // its first token and how many it has
  };
  // An item from its record and the raw count of its list (raw_count: one scalar load, nothing else, so
  // that the load can be requested well ahead of make_item).
  auto raw_count = [&](int rec) __attribute__((always_inline)) {
    typedef const int32_t __attribute__((address_space(4))) * const_i32_t;
    const int bh = rec / RSA_MAX_BLOCKS, qb = rec % RSA_MAX_BLOCKS;
    const bool sp = !dense_all && qb < dm.n;
    return sp ? ((const_i32_t)(uintptr_t)a.count)[(size_t)bh * dm.n + qb] : dm.m;
  };
  auto make_item = [&](int rec, int cnt) __attribute__((always_inline)) {
    Item it;
    it.bh = rec / RSA_MAX_BLOCKS;
    it.qb = rec % RSA_MAX_BLOCKS;
    const bool sp = !dense_all && it.qb < dm.n;
    const size_t vrow = (size_t)it.bh * dm.n + it.qb;
    it.nlist = min(max(cnt, 1), dm.m);        // as list_length() holds it
    it.ns = it.nlist * C::SPB;
    it.has_list = sp ? 1 : 0;
    const int b = it.bh / dm.heads, h = it.bh % dm.heads;
    const int64_t base = (int64_t)b * dm.sb + (int64_t)h * dm.sh;
    // (with RSA_DENSE every list pointer may be NULL: a dense row reads the first word of Q instead)
    it.list = (const_list_t)(uintptr_t)(sp ? (const void*)(a.block_idx + vrow * dm.m) : (const void*)a.Q);
    it.Kbytes = (uint64_t)(uintptr_t)(a.K + base);
    it.Vtbytes = (uint64_t)(uintptr_t)(a.Vt + (size_t)it.bh * dm.m * D * BLK);
    const int64_t t0 = dm.block_start(it.qb);
    it.q_t0 = (int)t0;
    it.q_count = dm.block_count(it.qb);
    it.qo_off = base + t0 * dm.st;
    return it;
  };
  auto load_item = [&](int k) __attribute__((always_inline)) {
    const int rec = my_record(k);
    return make_item(rec, raw_count(rec));
  };

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
  auto open_block = [&](int m, uint64_t Kbytes, uint64_t Vtbytes) __attribute__((always_inline)) {
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
  auto issue_load = [&](const Tile& t, auto idxc) __attribute__((always_inline)) {
    constexpr int idx = decltype(idxc)::value;
    if constexpr (idx < C::KPW) {
      constexpr int ii = idx;
      dma16_sv_imm<(ii / KOFF) * K_LDS_PASS + (ii % KOFF) * K_LDS_CLASS>(t.kdst, t.kp, kvw[ii], lds);
    } else {
      constexpr int ii = idx - C::KPW;
      dma16_sv_imm<(ii / VOFF) * V_LDS_PASS + (ii % VOFF) * V_LDS_CLASS>(t.vdst, t.vp, vvo[ii], lds);
    }
  };

  // ---- loop-invariant LDS read positions (16-byte chunk index inside stage 0, tile 0) ----
  const u32x4* kread[C::KS];
  const u32x4* vread[C::PC];
#pragma unroll
  for (int ks = 0; ks < C::KS; ++ks) kread[ks] = lds + swizzled<C::KCPR>(l32, 2 * ks + hf);
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) vread[pc] = lds + KSTAGES * KBUF + swizzled<C::VCPR>(l32, 2 * pc + hf);

  // ---- the item being computed, the one after it, and the one whose output is still to be written
  Item cur = {}, nxt = {};
  int nxt_valid = 0, k_next = 0;       // k_next: the first item not yet loaded
  int rec_ahead = 0;                   // ... and its record, read an item ahead
  // what the epilogue needs of the item that has just ended
  int done_bh = 0, done_sparse = 0, done_q_t0 = 0, done_q_count = 0;
  int64_t done_qo_off = 0;

  // Q as the B operand of S^T = K Q^T, resident in registers; the next item's rows replace it right
  // behind the last K Q^T of the current one.
  bf16x8 qreg[C::KS];
  const float cs = dm.scale * kLog2e;   // scores -> binades
  auto load_q = [&](const Item& it) __attribute__((always_inline)) {
    const int ln = lane_now();
    const int q = wave * 32 + ln % 32;
    const uint16_t* qrow = a.Q + it.qo_off + (int64_t)q * dm.st + 8 * (ln / 32);
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (q < it.q_count) v = *reinterpret_cast<const uint4*>(qrow + 16 * s);
      qreg[s] = __builtin_bit_cast(bf16x8, v);
    }
  };
  floatx16 oacc[C::DT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float mref = 0.f, lpart = 0.f;         // softmax reference (log2 domain) and this lane's partial row sum

  // Epilogue of one item: O = R_n * acc / l + C_n (video rows; text rows: acc / l), bf16; then the
  // running state starts over for the next item. R_n and C_n are requested a step ahead (in the
  // softmax phase of the item's last step): lane j holds elements CV*j .. CV*j+CV-1 of C_n, and every
  // lane collects the 64 it needs through the LDS crossbar -- no memory latency is left in here.
  constexpr int CV = D / 64;
  float done_comp[CV];
#pragma unroll
  for (int j = 0; j < CV; ++j) done_comp[j] = 0.f;
  float done_rfac = 1.0f;
  auto request_epilogue = [&](const Item& it) __attribute__((always_inline)) {
    const size_t vrow = (size_t)it.bh * dm.n + it.qb;          // row of the per-video-block tensors
    done_rfac = 1.0f;
    if (it.has_list && (a.flags & RSA_RECTIFY_CRITICAL)) {
      typedef const float __attribute__((address_space(4))) * const_f32_t;    // scalar load
      done_rfac = ((const_f32_t)(uintptr_t)a.R)[vrow];
    }
    if (it.has_list && (a.flags & RSA_COMPENSATE)) {
      const float* crow = a.comp + vrow * D + lane_now() * CV;
#pragma unroll
      for (int j = 0; j < CV; ++j) done_comp[j] = crow[j];
    }
  };
  auto settle_item_loads = [&]() __attribute__((always_inline)) {       // a use of everything load_q and request_epilogue asked for
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : "+v"(qreg[ks]));
#pragma unroll
    for (int j = 0; j < CV; ++j) asm volatile("" : "+v"(done_comp[j]));
  };
  auto write_output = [&]() __attribute__((always_inline)) {
    const bool do_comp = done_sparse && (a.flags & RSA_COMPENSATE);
    const int q_count = done_q_count;
    const float lsum = half_wave_sum(lpart);
    const int ln = lane_now();
    const int hf = ln / 32;                        // (a copy of its own: see lane_now)
    const int q = wave * 32 + ln % 32;
    const float f = done_rfac / lsum;
    uint16_t* orow = a.O + done_qo_off + (int64_t)q * dm.st;
    const int hf_lane4 = (4 * hf / CV) * 4;        // byte address of lane (4 hf)/CV for the crossbar
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) {
      // the 16 elements of C_n that go with this accumulator tile, all requested before the first is used
      // (element 32 dt + 8 g + 4 hf + e; every lane takes part: one outside the block still lends its share)
      float cadd[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) cadd[r] = 0.f;
      if (do_comp) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dc = 32 * dt + 8 * (r / 4) + (r % 4);        // + 4 hf: a multiple of CV
          const int c = __builtin_amdgcn_ds_bpermute(hf_lane4 + (dc / CV) * 4, __builtin_bit_cast(int, done_comp[dc % CV]));
          cadd[r] = __builtin_bit_cast(float, c);
        }
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d0 = 32 * dt + 8 * g + 4 * hf;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = fmaf(oacc[dt][4 * g + e], f, cadd[4 * g + e]);
        if (q < q_count) {
          uint2 w;
          w.x = pack_bf16x2(o[0], o[1]);
          w.y = pack_bf16x2(o[2], o[3]);
          *reinterpret_cast<uint2*>(orow + d0) = w;
        }
      }
    }
    if (q < q_count && a.lse && hf == 0)
      a.lse[((size_t)done_bh * dm.t) + done_q_t0 + q] = (mref + log2f(lsum)) * 0.6931471805599453f;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    mref = 0.f;
    lpart = 0.f;
  };

  // Two groups of waves share every SIMD (wave w of group 0 and wave w of group 1). They run
  // the same sequence  [M(s) | barrier | V(s) | barrier] ...  one barrier apart, so that while
  // one group issues MFMAs the other does its softmax on the VALU. s counts the steps of all the
  // items of the group, one after the other without a gap:
  //   M(s): O^T += V^T P^T of step s-1, then S^T = K Q^T of step s: matrix instructions only, the A
  //         operand of each read from LDS a few slots ahead (V^T tile of step s-1 from its ring
  //         stage (s-1) % 3, K tile of step s from stage s % 2); the loads of tile s+1 (K into
  //         stage (s+1) % 2, V^T into stage (s+1) % 3) go out one per MFMA slot. Behind the last
  //         step of an item the query rows of the next item are requested.
  //   V(s): in the first step of an item, the output of the item before it; mask, online softmax
  //         -> P as bf16 B operands (VALU only); fetch the list entry of step s+2; wait for tile
  //         s+1; read the first V^T operands of M(s+1) ahead of the barrier
  // The barrier after V(s) publishes tile s+1 to the group. A K stage is rewritten two steps
  // after it was read, a V^T stage (read in M(s+1), one phase after its K tile) three steps after
  // it was filled: by then every wave of the group has passed the barrier that follows its last
  // read. Every item has an even number of steps (SPB = 2 per key block), so the position inside a
  // key block and the K stage both follow from the parity of s, which the unrolled loop knows.
  int m_nxt_e = 0, m_nxt_j = 0;   // key block that the next new-block step opens: entry m_nxt_e of a list, or block m_nxt_j (>= 0) of a dense row
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
  Tile vt_next = {};          // the tile of step s+1 as M(s) prepared it: its V^T rows are requested in V(s)
  const u32x4* vcur[C::PC];   // vread[] moved to the V^T stage whose P V product comes next
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) vcur[pc] = vread[pc];
  auto read_v_operand = [&](int slot) __attribute__((always_inline)) {      // slot < NPV
    const int pc = slot / C::DT, dt = slot % C::DT;
    ring[slot % W] = __builtin_bit_cast(bf16x8, vcur[pc][dt * 32 * C::VCPR]);
  };

  // Variants of the two phases, all compile-time:
  //   MFMA phase  QK: 0 = the last P V product of the group alone.  LAST: the step is the last of its item
  //               -- the tile of step s+1 may open the next item (that item's K and V^T), and the next
  //               item's query rows are requested behind the last K Q^T.
  //   softmax phase  FIRST: first step of an item (the output of the item before it is written first);
  //               FETCH: 0 none (odd steps), 1 the next entry of the item's own list, 2 wherever step
  //               s+2 falls (own list, first entry of the next item, or the last entry once more);
  //               LAST: behind it the next item takes the place of the current one.
  // The steps in the middle of an item run the plain variants in a loop of their own, so that what
  // only the boundaries between items need stays out of its registers.
  auto m_phase = [&](auto stc, auto qkc, auto lastc) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;          // s modulo 2: the K stage and the part of the key block
    constexpr bool do_qk = decltype(qkc)::value != 0, last_of_item = decltype(lastc)::value != 0;
    constexpr int DSLOT = RSA_DSLOT;                  // the slot in which the requests for the next tile start
    constexpr int MLOADS = SPLIT_LOADS ? C::KPW : LPS;   // requests of this phase: the K rows, or the whole tile
    constexpr int LAST = do_qk ? NSLOT : NPV;         // slots that hold an MFMA
    constexpr int WB = W / 2;                         // operands are waited for WB at a time
    Tile nt = {};
    // The wave that feeds the matrix pipe goes first wherever the two waves of a SIMD compete for an
    // issue slot: without this the older wave of the two wins, and the MFMA phases of the younger
    // group run a fifth longer than those of the other.
    __builtin_amdgcn_s_setprio(3);
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, LAST>([&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      // The operands of slots i .. i+WB-1 have arrived once at most the reads behind them are
      // outstanding: one wait per WB slots, and none is needed in between.
      if constexpr (i % WB == 0) {
        constexpr int behind = (LAST - i - WB) < 0 ? 0 : ((LAST - i - WB) < (W - WB) ? (LAST - i - WB) : (W - WB));
        // vmcnt and expcnt fields at "no wait", lgkmcnt = behind
        __builtin_amdgcn_s_waitcnt(0xC07F | (behind << 8));
        __builtin_amdgcn_sched_barrier(0);
      }
      // one load of the tile of step s+1 per slot, behind the MFMA of the slot before
      if constexpr (do_qk && i >= DSLOT && i - DSLOT < MLOADS) issue_load(nt, IntC<i - DSLOT>{});
      if constexpr (i < NPV) {
        constexpr int pc = i / C::DT, dt = i % C::DT;
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % W], __builtin_bit_cast(bf16x8, pb[pc]), oacc[dt], 0, 0, 0);
      } else {
        constexpr int q = i - NPV, k2 = q / C::KT, t = q % C::KT;
        floatx16 c0 = sacc[t];
        if constexpr (k2 == 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) c0[r] = 0.f;           // folds into the instruction's constant C operand
        }
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % W], qreg[k2], c0, 0, 0, 0);
      }
      // the ring entry this slot used takes the operand of slot i + W
      if constexpr (i + W < LAST) {
        constexpr int slot = i + W;
        if constexpr (slot < NPV) {
          read_v_operand(slot);
        } else {
          constexpr int q = slot - NPV, k2 = q / C::KT, t = q % C::KT;
          ring[slot % W] = __builtin_bit_cast(bf16x8, kread[k2][(ST % KSTAGES) * KBUF + t * 32 * C::KCPR]);
        }
      }
      if constexpr (do_qk && i < 2) {
        // behind the first MFMAs, so that the matrix pipe starts as soon as the barrier opens:
        // addresses of the tile of step s+1. Whether that step opens a new key block (its list entry
        // came in during V(s-1)) follows from the parity of s. A group whose last step this is
        // requests the tile of its last list entry once more, into a stage nobody reads again.
        __builtin_amdgcn_sched_barrier(0);
        constexpr int PART_NEXT = (ST + 1) % C::SPB;
        if constexpr (i == 0) {
          if constexpr (PART_NEXT == 0) {
            const bool in_next = last_of_item && nxt_valid;
            open_block(m_nxt_j >= 0 ? m_nxt_j : m_nxt_e, in_next ? nxt.Kbytes : cur.Kbytes, in_next ? nxt.Vtbytes : cur.Vtbytes);
          }
          kvc_nxt = blk_count;
        } else {
          step_of_block(nt, PART_NEXT, (ST + 1) % KSTAGES, vst + 1 >= VSTAGES ? 0 : vst + 1);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // a phase with fewer slots than loads sends the rest here
    static_for<0, MLOADS>([&](auto ic) __attribute__((always_inline)) {
      constexpr int idx = decltype(ic)::value;
      if constexpr (do_qk && DSLOT + idx >= LAST) issue_load(nt, ic);
    });
    if constexpr (do_qk) vt_next = nt;
    if constexpr (SPLIT_LOADS) {
      // the V^T rows of this step (requested a phase ago, ahead of this phase's K rows) have landed
      wait_loads_leaving<do_qk ? MLOADS : 0>();
    }
    // behind the last K Q^T of an item: the query rows of the next one (they arrive before the end of
    // the softmax phase, which waits for every load)
    if constexpr (do_qk && last_of_item) {
      if (nxt_valid) load_q(nxt);
    }
  };

  // entry j of an item's list; a dense row: j itself
  auto list_entry = [&](const Item& it, int j) __attribute__((always_inline)) {
    const int e = it.list[it.has_list ? j : 0];
    return it.has_list ? e : j;
  };

  int fj = 0;                 // entry of the current item's list that the next even step fetches
  int have_output = 0;        // an item has ended and its output is still in the accumulators
  auto v_phase = [&](auto stc, auto firstc, auto fetchc, auto lastc) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;
    constexpr bool first_of_item = decltype(firstc)::value != 0, last_of_item = decltype(lastc)::value != 0;
    constexpr int FETCH = decltype(fetchc)::value;
    __builtin_amdgcn_s_setprio(0);
    constexpr int VLOADS = SPLIT_LOADS ? C::VPW : 0;  // requests of this phase: the V^T rows of step s+1
    // The last step of an item: what the switch to the next item and the epilogue need from memory is
    // requested here, a whole softmax ahead of its use -- R_n and C_n of this item, the list length of
    // the item after the next (its record came in an item ago), the record of the one after that.
    int cnt_ahead = 0, rec_new = 0;
    bool more = false;
    if constexpr (last_of_item) {
      request_epilogue(cur);
      more = k_next < n_my_items;
      if (more) cnt_ahead = raw_count(rec_ahead);
      if (k_next + 1 < n_my_items) rec_new = my_record(k_next + 1);
    }
    // The list entry of step s+2 (an even step opens a key block) for M(s+1): requested ahead of the
    // softmax, which hides the scalar cache miss that every sixteenth entry (and the head of every list)
    // is. Only the load is here -- what the entry means (a dense row has none: its j-th block is j)
    // is settled where M(s+1) opens the block.
    if constexpr (FETCH == 1) {
      m_nxt_e = cur.list[cur.has_list ? fj : 0];
      m_nxt_j = cur.has_list ? -1 : fj;
      fj += 1;
    } else if constexpr (FETCH == 2) {
      // it may be the first entry of the next item; past the last item, the last entry again (a valid
      // block: the tile requested for a step that does not exist is never read)
      const bool own = fj < cur.nlist, follow = !own && nxt_valid;
      const_list_t lp = follow ? nxt.list : cur.list;
      const int hl = follow ? nxt.has_list : cur.has_list;
      const int j = own ? fj : (follow ? 0 : cur.nlist - 1);
      m_nxt_e = lp[hl ? j : 0];
      m_nxt_j = hl ? -1 : j;
      fj += 1;
    }
    if constexpr (SPLIT_LOADS && !first_of_item) {
      static_for<0, C::VPW>([&](auto ic) __attribute__((always_inline)) { issue_load(vt_next, IntC<C::KPW + decltype(ic)::value>{}); });
    }
    // the first step of an item: the P V products of the item before it are complete
    // (tile s+1 is waited for first: the loads of the output would otherwise be waited for together
    // with it at the end of the phase, and so would the stores, which now complete under the next
    // MFMA phase)
    if constexpr (first_of_item) {
      if (have_output) {
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
        write_output();
      }
      if constexpr (SPLIT_LOADS) {
        static_for<0, C::VPW>([&](auto ic) __attribute__((always_inline)) { issue_load(vt_next, IntC<C::KPW + decltype(ic)::value>{}); });
      }
    }
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
      // Scores are counted in binades (score * scale * log2 e) from a reference that starts at 0 for
      // every item and moves rarely: fp32 sums and bf16 operands span 2^+-126, so probabilities may
      // sit anywhere within 2^+-kLazyBits of one another's scale. No maximum is taken on the way: the
      // probabilities of the step are worked out against the current reference, and only when their
      // sum says that one of them left the window (above it; in the first step of an item, all of
      // them below it, too) is the step done again the long way -- the scores are still in registers
      // -- with the row maximum as the new reference and everything gathered so far rescaled.
      constexpr float kAbove = 1.0995116e12f, kBelow = 9.0949470e-13f;        // 2^+-kLazyBits
      static_assert(kLazyBits == 40.0f, "kAbove and kBelow are 2^+-kLazyBits");
      auto probabilities = [&]() __attribute__((always_inline)) {
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < C::KT; ++t) {
          float p[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[t][r], cs, -mref));
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            u32x4 w;
            w.x = pack_bf16x2(p[8 * u + 0], p[8 * u + 1]);
            w.y = pack_bf16x2(p[8 * u + 2], p[8 * u + 3]);
            w.z = pack_bf16x2(p[8 * u + 4], p[8 * u + 5]);
            w.w = pack_bf16x2(p[8 * u + 6], p[8 * u + 7]);
            pb[2 * t + u] = w;
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += p[8 * u + i];
          }
        }
        return sum;
      };
      float rs = probabilities();
      bool outside = rs > kAbove;
      if constexpr (first_of_item) outside = outside || rs < kBelow;
      if (__any(outside)) {
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < C::KT; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][r]);
        mx = half_wave_max(mx) * cs;                   // the scale is positive
        if constexpr (first_of_item) {
          mref = mx;                                   // accumulators and row sum are empty: nothing to rescale
        } else {
          const float mnew = fmaxf(mref, mx);
          const float alpha = __builtin_amdgcn_exp2f(mref - mnew);
          mref = mnew;
          lpart *= alpha;
#pragma unroll
          for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
        }
        rs = probabilities();
      }
      lpart += rs;
    }
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
    if constexpr (last_of_item) {
      // the item has ended: its output waits for the last P V product; the next item takes its place
      done_bh = cur.bh;
      done_sparse = cur.has_list;
      done_q_t0 = cur.q_t0;
      done_q_count = cur.q_count;
      done_qo_off = cur.qo_off;
      have_output = 1;
      if (nxt_valid) {
        cur = nxt;
        fj = 1;                          // entry 0 was fetched two steps ago
        nxt_valid = more;
        if (more) nxt = make_item(rec_ahead, cnt_ahead);
        rec_ahead = rec_new;
        k_next += 1;
      }
    }
    // tile s+1 has landed (this wave's share; the barrier that follows covers the group), and so
    // have the query rows of the next item
    // (loads return in order: only this phase's own requests may still be out)
    if constexpr (first_of_item) {
      if (!have_output) wait_loads_leaving<VLOADS>();
    } else {
      wait_loads_leaving<VLOADS>();
    }
    if constexpr (last_of_item) {
      // The compiler waits for the loads it knows of (the query rows, C_n) where they are first used, and
      // such a wait covers the tile requests as well: it belongs here, where the youngest request is a
      // whole phase old, not behind the first requests of the next MFMA phase.
      settle_item_loads();
    }
  };

  const bool active = n_my_items > 0;
  if (active) {
    cur = load_item(0);
    nxt_valid = n_my_items > 1;
    if (nxt_valid) nxt = load_item(1);
    k_next = 2;
    if (n_my_items > 2) rec_ahead = my_record(2);
    load_q(cur);
    // Q must have arrived before the first direct-to-LDS load is requested: the compiler
    // does not see those loads, and would otherwise place its own wait for Q -- a wait for
    // *every* outstanding load -- at the first use inside the loop.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    Tile t0;
    open_block(list_entry(cur, 0), cur.Kbytes, cur.Vtbytes);
    step_of_block(t0, 0, 0, 0);
    static_for<0, LPS>([&](auto ic) __attribute__((always_inline)) { issue_load(t0, ic); });
    kvc_cur = blk_count;
    fj = 1;
    // The first MFMA phase multiplies the (zero) probabilities of a step that does not exist with
    // whatever the last V^T stage holds: make that zeros too (0 x NaN would poison the accumulators).
    {
      u32x4* vlast = lds + KSTAGES * KBUF + (VSTAGES - 1) * C::VBUF;
      for (int c = wave * 64 + lane; c < C::VBUF; c += C::NW * 64) vlast[c] = u32x4{0u, 0u, 0u, 0u};
      // ... and the operands read ahead of it come from there
#pragma unroll
      for (int pc = 0; pc < C::PC; ++pc) vcur[pc] = vread[pc] + (VSTAGES - 1) * C::VBUF;
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  group_barrier();                  // tile 0 of every group is in LDS
  if (active) {
#pragma unroll
    for (int j = 0; j < W; ++j) read_v_operand(j);
  }
  if (grp >= NGRP / 2) group_barrier();    // the second half of the groups runs one barrier behind the first
  // Every group turns wg_rounds rounds of two barriers; round s is M(s), V(s) while the group has
  // steps left, the last P V product and the last output in round my_total, and nothing but the
  // barriers after.
  using Y = IntC<1>;
  using N = IntC<0>;
  int s = 0;
  if (active) {
    for (int item = 0; item < n_my_items; ++item) {
      const int ns = cur.ns;
      // step 0 of the item
      m_phase(IntC<0>{}, Y{}, N{});
      group_barrier();
      v_phase(IntC<0>{}, Y{}, IntC<2>{}, N{});
      group_barrier();
      if (ns >= 4) {
        // steps 1 .. ns-4 in pairs: nothing but this item's own list and tiles
        for (int sj = 1; sj + 3 < ns; sj += 2) {
          m_phase(IntC<1>{}, Y{}, N{});
          group_barrier();
          v_phase(IntC<1>{}, N{}, IntC<0>{}, N{});
          group_barrier();
          m_phase(IntC<0>{}, Y{}, N{});
          group_barrier();
          v_phase(IntC<0>{}, N{}, IntC<1>{}, N{});
          group_barrier();
        }
        // steps ns-3 and ns-2: the latter fetches the first list entry of the next item
        m_phase(IntC<1>{}, Y{}, N{});
        group_barrier();
        v_phase(IntC<1>{}, N{}, IntC<0>{}, N{});
        group_barrier();
        m_phase(IntC<0>{}, Y{}, N{});
        group_barrier();
        v_phase(IntC<0>{}, N{}, IntC<2>{}, N{});
        group_barrier();
      }
      // step ns-1
      m_phase(IntC<1>{}, Y{}, Y{});
      group_barrier();
      v_phase(IntC<1>{}, N{}, IntC<0>{}, Y{});
      group_barrier();
      s += ns;
    }
    m_phase(IntC<0>{}, N{}, N{});
    group_barrier();
    __builtin_amdgcn_s_setprio(0);
    write_output();
    // nothing may be in flight into the LDS of a workgroup that is about to end
    __builtin_amdgcn_s_waitcnt(0x0F70);
    group_barrier();
    s += 1;
  }
  for (; s < wg_rounds; ++s) {
    group_barrier();
    group_barrier();
  }
  if (grp < NGRP / 2) group_barrier();
}

template <int D, int BLK>
hipError_t launch_attn_t(const Dims& dm, const AttnArgs& a, const AttnSched& ws, hipStream_t s) {
  using C = AttnCfg<D, BLK>;
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int n_wg = ws.n_wg;
  if (n_wg < 8 || n_wg % 8) return hipErrorInvalidValue;
  const SchedShape sh = sched_shape(dm, a.flags, n_wg, C::NGRP);
  SchedArgs sc = {};
  sc.n_items = sh.n_items;
  sc.n_dense = sh.n_dense;
  sc.dense_per_bh = sh.dense_per_bh > 0 ? sh.dense_per_bh : 1;
  sc.dense_first = sh.dense_first;
  const bool compensate = !dense_all && (a.flags & RSA_COMPENSATE);
  const bool deal = ws.table && sh.n_queues * 64 <= RSA_ATTN_SCHED_SLOTS && (size_t)sh.n_queues * 64 * sh.cap <= ws.table_entries;
  DealArgs da = {};
  if (deal) {
    da.table = ws.table; da.nitems = ws.nitems; da.total = ws.total;
    da.cap = sh.cap; da.n_queues = sh.n_queues; da.slots_per_xcd = sh.slots_per_xcd;
    da.n_dense = sh.n_dense; da.dense_per_bh = sc.dense_per_bh; da.dense_first = sh.dense_first;
    sc.table = ws.table; sc.nitems = ws.nitems; sc.total = ws.total; sc.cap = sh.cap;
  }
  const hipError_t side = launch_attn_side(dm, a, da, !dense_all && a.row_order, compensate, deal, C::SPB, s);
  if (side != hipSuccess) return side;
  hipLaunchKernelGGL((attn_kernel<D, BLK>), dim3((unsigned)n_wg), dim3(C::NTHR), 0, s, dm, a, sc);
  return hipGetLastError();
}

}  // namespace

// Entries of the schedule table for RSA_ATTN_MAX_WGS resident workgroups, dense launch or not. (A GPU
// with fewer CUs forms fewer, longer queues; should its table not fit, the items go out in index order.)
size_t attn_sched_entries(const Dims& dm) {
  const int ngrp = dm.blk == 128 ? 2 : 4;
  size_t need = 0;
  for (int flags : {0, (int)RSA_DENSE}) {
    const SchedShape sh = sched_shape(dm, flags, RSA_ATTN_MAX_WGS, ngrp);
    const size_t e = (size_t)sh.n_queues * 64 * (size_t)sh.cap;
    need = e > need ? e : need;
  }
  return need;
}

hipError_t launch_attn(const Dims& dm, const AttnArgs& a, const AttnSched& ws, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_attn_t<128, 128>(dm, a, ws, s);
  if (dm.d == 128 && dm.blk == 64) return launch_attn_t<128, 64>(dm, a, ws, s);
  if (dm.d == 64 && dm.blk == 128) return launch_attn_t<64, 128>(dm, a, ws, s);
  return launch_attn_t<64, 64>(dm, a, ws, s);
}

}  // namespace rsa
