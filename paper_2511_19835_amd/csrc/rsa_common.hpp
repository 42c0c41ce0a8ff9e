// Shared declarations of the librsa.so translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rsa.h"

namespace rsa {

// Sizes derived from an rsa_shape; passed by value to every kernel.
struct Dims {
  int batch, heads, d, blk;
  int64_t tv, tt, t;     // T_v, T_t, T
  int n;                 // N: video blocks
  int mt;                // text blocks
  int m;                 // M = N + mt
  int w;                 // mask words per row
  int64_t sb, sh, st;    // element strides of Q/K/V/O
  float scale;

  __host__ __device__ inline int64_t block_start(int blk_idx) const {
    return blk_idx < n ? (int64_t)blk_idx * blk : tv + (int64_t)(blk_idx - n) * blk;
  }
  __host__ __device__ inline int block_count(int blk_idx) const {
    int64_t rem = blk_idx < n ? tv - (int64_t)blk_idx * blk : tt - (int64_t)(blk_idx - n) * blk;
    return rem < blk ? (int)rem : blk;
  }
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}
// Round-to-nearest-even pair conversion (v_cvt_pk_bf16_f32): low half = a, high half = b.
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  floatx2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
__device__ inline uint16_t to_bf16_bits(float a) { return (uint16_t)(pack_bf16x2(a, 0.f) & 0xffffu); }

// fp16 (round-to-nearest-even), saturated to the largest finite half so that an out-of-range
// value stays finite: the operands of the gate GEMMs carry 11 significant bits instead of 8.
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
__device__ inline uint32_t pack_f16x2_sat(float a, float b) {
  floatx2 f = {fminf(fmaxf(a, -65504.f), 65504.f), fminf(fmaxf(b, -65504.f), 65504.f)};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, halfx2));
}
__device__ inline uint16_t to_f16_bits_sat(float a) { return (uint16_t)(pack_f16x2_sat(a, 0.f) & 0xffffu); }

// fp16 copies of the pooled vectors, laid out as the B operand of the gate GEMMs reads them:
// vectors in groups of 32; for group g and k-step s (16 channels) the 64 lanes of a wave read
// 1 KB in one piece -- lane = 32*hf + l32 holds channels 16s + 8hf .. +7 of vector 32g + l32.
// Half-precision element offset of (vector o, channel c) inside one (batch, head):
template <int D>
__host__ __device__ inline size_t gate_operand_offset(int o, int c) {
  return ((((size_t)(o / 32) * (D / 16) + c / 16) * 2 + (c % 16) / 8) * 32 + o % 32) * 8 + c % 8;
}
// Adds the eight bf16 values of a 16-byte chunk to eight running sums (the block-mean reduction).
__device__ inline void accumulate8(float (&acc)[8], const uint4& v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += bf16_bits_to_float(w[i] & 0xffffu);
    acc[2 * i + 1] += bf16_bits_to_float(w[i] >> 16);
  }
}
// vectors are padded to a multiple of 32 per (batch, head)
__host__ __device__ inline size_t gate_operand_vectors(int n) { return (size_t)((n + 31) / 32) * 32; }

// ---- launchers (one per translation unit) -------------------------------------------
struct PoolArgs {
  const uint16_t *Q, *K, *V;
  float *Qp, *Kp, *Vp;
  uint16_t* Vt;
  uint16_t *Qpb, *Kpb;     // optional fp16 copies of the pooled vectors in gate_operand_offset layout
  bool skip_k = false;     // the pooled keys come from the key-side launch of the gate (launch_gapr_keys)
  // when both are set (and Q is pooled by this call: the pooled queries are needed), the launch that pools V also
  // writes the text columns of Lmass from the text keys of text_K
  const uint16_t* text_K = nullptr;
  float* text_Lmass = nullptr;
};
hipError_t launch_pool(const Dims& dm, const PoolArgs& a, hipStream_t s);

struct ScoreArgs {
  const uint16_t* K;
  const float *Qp, *Kp;
  float *Spool, *Apool, *Lmass;
  bool text_done = false;  // the text columns of Lmass are already written (by the launch that pooled V)
};
hipError_t launch_scores(const Dims& dm, const ScoreArgs& a, hipStream_t s);

struct GaprArgs {
  const uint16_t *Q, *K;
  const float *Qp, *Kp;    // fp32 pooled vectors (the centre of each token block)
  const uint16_t *Qpb, *Kpb;
  const float* Spool;
  float* DBt;              // key-side deviations, [b][h][M][N] (workspace)
  uint32_t* Mc_bits;
  int mode;
  float* Kp_out = nullptr;       // launch_gapr_keys: pooled keys, written by the launch that reads the key blocks anyway
  uint16_t* Kpb_out = nullptr;
};
// mode 1 is two launches with the pooled scores between them: the key side (needs Qpb; writes DBt and, when
// Kp_out is set, the pooled keys) and the query side (needs Kpb, Spool, DBt; writes Mc_bits). launch_gapr runs
// both (pooled keys given), or fills Mc_bits for the other modes.
hipError_t launch_gapr_keys(const Dims& dm, const GaprArgs& a, hipStream_t s);
hipError_t launch_gapr_queries(const Dims& dm, const GaprArgs& a, hipStream_t s);
hipError_t launch_gapr(const Dims& dm, const GaprArgs& a, hipStream_t s);

struct SelectArgs {
  const float *Lmass, *Apool;
  const uint32_t* forced;
  uint32_t* mask_bits;
  int32_t *block_idx, *count;
  float* R;
  int keep;
  float p;
};
hipError_t launch_select(const Dims& dm, const SelectArgs& a, hipStream_t s);

hipError_t launch_adjacency(const Dims& dm, const int* grid, const int* tile, int radius, uint32_t* bits,
                            hipStream_t s);

hipError_t launch_reorder(const Dims& dm, const int* grid, const int* tile, int direction, const uint16_t* src,
                          uint16_t* dst, hipStream_t s);

struct AttnArgs {
  const uint16_t *Q, *K, *Vt;
  const int32_t *block_idx, *count;
  const uint32_t *mask_bits, *Mc_bits;
  const float *R, *Apool, *Vp;
  uint16_t* O;
  float* lse;
  float* comp;             // workspace [b][h][N][d]: pooled compensation term C_n
  int32_t* row_order;      // workspace [b][h][N]: launch order of the video query blocks (NULL: natural)
  int flags;
};
// Persistent attention kernel: number of resident workgroups and (optional) room for its schedule.
#define RSA_ATTN_MAX_WGS 256
struct AttnSched {
  int n_wg;                 // workgroups to launch: a multiple of 8, at most RSA_ATTN_MAX_WGS
  int32_t* table;           // NULL: items are dealt in index order
  int32_t *nitems, *total;  // [RSA_ATTN_SCHED_SLOTS] each
  size_t table_entries;     // room in `table`
};
#define RSA_ATTN_SCHED_SLOTS 4096
size_t attn_sched_entries(const Dims& dm);   // table entries that rsa_workspace_bytes sets aside
hipError_t launch_attn(const Dims& dm, const AttnArgs& a, const AttnSched& ws, hipStream_t s);

}  // namespace rsa
