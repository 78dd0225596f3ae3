// Shared host/device helpers of the lshe HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lshe.h"

namespace lshe {

constexpr int kWave = 64;
constexpr int kMaxBudget = 1 << 20;   // slot index must fit the low 20 bits of a selection key
constexpr int kMaxGroup = 16;

// ---- problem sizes derived from a validated config ---------------------------------------
struct Dims {
  int d, r, W, H, G, L, B, C, dtype, n_sink, n_recent, policy;
  int Wr;      // code words of the projection matrix (ceil(r/32)); W is words per SLOT code
  int64_t units;
  int esize;   // bytes per element of K/V/Q/out
};

inline int validate(const lshe_config *c) {
  if (!c) return LSHE_INVALID_ARG;
  if (c->hash_bits < 1 || c->hash_bits > 64) return LSHE_INVALID_ARG;
  if (c->n_kv_heads < 1 || c->n_layers < 1 || c->batch < 1) return LSHE_INVALID_ARG;
  if (c->gqa_group < 1 || c->gqa_group > kMaxGroup) return LSHE_INVALID_ARG;
  if (c->budget < 1 || c->budget >= kMaxBudget) return LSHE_INVALID_ARG;
  if (c->dtype != LSHE_F32 && c->dtype != LSHE_BF16) return LSHE_INVALID_ARG;
  if (c->n_sink < 0 || c->n_recent < 0) return LSHE_INVALID_ARG;
  if (c->policy != LSHE_POLICY_HASH && c->policy != LSHE_POLICY_L2NORM) return LSHE_INVALID_ARG;
  if ((int64_t)c->n_sink + (int64_t)c->n_recent >= (int64_t)c->budget) return LSHE_INVALID_ARG;
  if (c->head_dim < 1) return LSHE_INVALID_ARG;
  if (c->head_dim != 64 && c->head_dim != 128) return LSHE_UNSUPPORTED;
  int64_t units = (int64_t)c->batch * c->n_layers * c->n_kv_heads;
  if (units > (int64_t)1 << 24) return LSHE_UNSUPPORTED;
  return LSHE_OK;
}

inline Dims dims_of(const lshe_config *c) {
  Dims m;
  m.policy = c->policy;
  m.d = c->head_dim; m.r = c->hash_bits; m.Wr = (c->hash_bits + 31) / 32;
  m.W = c->policy == LSHE_POLICY_L2NORM ? 1 : (c->hash_bits + 31) / 32;
  m.H = c->n_kv_heads; m.G = c->gqa_group; m.L = c->n_layers; m.B = c->batch;
  m.C = c->budget; m.dtype = c->dtype; m.n_sink = c->n_sink; m.n_recent = c->n_recent;
  m.units = (int64_t)c->batch * c->n_layers * c->n_kv_heads;
  m.esize = c->dtype == LSHE_BF16 ? 2 : 4;
  return m;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- decode-attention work split (host decides, kernels are told) ------------------------
// Each unit's occupied slots are cut into `splits` contiguous chunks, one workgroup each;
// with more than one chunk a second small kernel merges the partial softmax states.
constexpr int kAttnThreads = 256;
constexpr int kAttnMinRows = 64;         // fewest slots worth a workgroup of their own
constexpr int kAttnTargetGroups = 256;   // workgroups wanted: one per CU (more, smaller ones cost
                                         // more in per-workgroup set-up, merge and partials than
                                         // they gain: 8 units x 9830 slots ran 33 us per step with
                                         // 1232 workgroups, 20 us with 256)

// Up to this many slot ranges per unit the whole-step form of the split plan merges with one
// small barrier-free workgroup per (unit, query head); above it with a workgroup of 1024 threads.
constexpr int kMergeSmallRanges = 32;

inline int attn_splits(int64_t units, int C) {
  int64_t want = (kAttnTargetGroups + units - 1) / units;
  int64_t cap = (C + kAttnMinRows - 1) / kAttnMinRows;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return (int)want;
}

// Launch plan of a decode step: with at least this many units (half the chip's 256 CUs), or
// with budgets so small that a step is launch-bound, one workgroup per unit runs the whole
// step in a single kernel; otherwise units are split over several workgroups (two kernels for a
// whole step, select + attention + merge for the stage-wise calls).
constexpr int kFusedMinUnits = 128;
constexpr int kFusedSmallBudget = 512;   // a unit this small is one workgroup's work anyway
// Groups of 8 query heads are the exception: one workgroup would carry 8 softmax states per
// lane (about 290 registers, one wave per SIMD), so beyond the launch-bound budgets their
// attention runs as two workgroups per unit with 4 query heads each (kernel after the select).
inline bool decode_is_fused(int64_t units, int C, int G) {
  if (G == 8 && C > kFusedSmallBudget) return false;
  return units >= kFusedMinUnits || C <= kFusedSmallBudget;
}

// Form of the single-kernel plan.  With fewer than kFusedManyUnits units (about one workgroup
// per CU) and a head that leaves a wave 256 registers, workgroups have 8 waves, else 4.  In
// the 8-wave form, when the unit's code table is small enough for one wave to score from
// registers (and long enough to be worth it), wave 0 selects alone while the others stream.
constexpr int kFusedManyUnits = 1024;
constexpr int kSoloMaxWords = 4096;   // code words per unit: 16 vectors of 16 bytes per lane
constexpr int kSoloMinBudget = 1024;  // below this the stream is too short to hide a select behind
inline bool fused_has_8_waves(const Dims &m) {
  return m.d == 128 && m.G * (m.dtype == LSHE_BF16 ? 1 : 2) <= 4 && m.units < kFusedManyUnits;
}
inline bool fused_select_is_solo(const Dims &m) {
  const int64_t words = (int64_t)m.C * m.W;   // a multiple of 4 keeps every unit's table 16-byte aligned
  return fused_has_8_waves(m) && m.C >= kSoloMinBudget && words <= kSoloMaxWords && words % 4 == 0;
}

// Workspace: the first 256-byte block holds the status word (bits that kernels OR in when a
// bounded internal wait expires; see lshe.h), every layout starts after it.
constexpr size_t kWsHeaderBytes = 256;
// Workspace of a decode step: partial softmax states per (unit, slot range) -- G x (d+2) floats
// ([max, sum, unnormalised output] per query head) for lshe_decode_attend --, then units x G
// floats that carry the victim's logit from the select kernel to the end of the attention
// (lshe_decode_select + lshe_decode_attend, groups of 8 heads on many units).
// (sized for the whole-step form of the split plan, which keeps two states per range, the set-aside
// row's logits and the range's selection key: local_part_floats)
__host__ __device__ inline int local_part_floats(int G, int HD) { return (2 * G * (HD + 2) + G + 2 + 3) & ~3; }
inline size_t decode_ws_partial_bytes(const Dims &m) {
  int S = attn_splits(m.units, m.C);
  return align_up((size_t)m.units * S * local_part_floats(m.G, m.d) * 4, 256);
}
// ... then 4 words per unit that carry the occupied-slot count, the token index and the new
// key's code from the attention kernel to the merge kernel of the split plan.
inline size_t decode_ws_logit_bytes(const Dims &m) { return align_up((size_t)m.units * m.G * 4, 256); }
inline size_t decode_ws_bytes(const Dims &m) {
  return kWsHeaderBytes + decode_ws_partial_bytes(m) + decode_ws_logit_bytes(m) +
         align_up((size_t)m.units * 16, 256);
}
// Workspace layout of a prefill: [header][codes_k: units x N x W][codes_q: units x G x (N-C) x W]
inline size_t prefill_ws_bytes(const Dims &m, int64_t N) {
  if (N <= 0) return 0;
  size_t nk = (size_t)m.units * (size_t)N * m.W * 4;
  size_t nq = N > m.C ? (size_t)m.units * m.G * (size_t)(N - m.C) * m.W * 4 : 0;
  return kWsHeaderBytes + align_up(nk, 256) + align_up(nq, 256);
}

#define LSHE_HIP_TRY(expr)                       \
  do {                                           \
    hipError_t e_ = (expr);                      \
    if (e_ != hipSuccess) return LSHE_HIP_ERROR; \
  } while (0)

#ifdef __HIPCC__
// ---- device helpers -----------------------------------------------------------------------

// Wall-clock stamps for an instrumented build (-DLSHE_STAMPS: lane 0 of every wave stores the
// constant-rate counter at numbered points of a kernel); compiled out otherwise.
#ifdef LSHE_STAMPS
constexpr int kStampSlots = 16, kStampWaves = 16, kStampGroups = 4096;
static __device__ unsigned long long g_stamps[kStampGroups][kStampWaves][kStampSlots];   // one copy per source file
#define LSHE_STAMP(k)                                                                         \
  do {                                                                                        \
    if ((threadIdx.x & 63) == 0 && blockIdx.x < lshe::kStampGroups)                           \
      lshe::g_stamps[blockIdx.x][threadIdx.x >> 6][k] = __builtin_amdgcn_s_memrealtime();     \
  } while (0)
#else
#define LSHE_STAMP(k) do { } while (0)
#endif

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// round-to-nearest-even float -> bf16 bits (finite inputs; NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wave, which would drain a stream of prefetches that the
// code on the far side of the barrier does not depend on; data handed over through LDS needs
// only the LDS counter to reach zero.  (Registers that a pending global load will fill stay
// tracked by the compiler's own wait insertion.)
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// DPP controls (GCN3+/CDNA encoding)
constexpr int kDppQuadSwap1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7-i inside each 8
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15-i inside each 16

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// max over the 16 lanes of a DPP row, result in every lane of the row
__device__ __forceinline__ uint32_t row16_max_u32(uint32_t x) {
  uint32_t y;
  y = dpp_u32<kDppQuadSwap1>(x); x = x > y ? x : y;
  y = dpp_u32<kDppQuadSwap2>(x); x = x > y ? x : y;
  y = dpp_u32<kDppRowHalfMirror>(x); x = x > y ? x : y;
  y = dpp_u32<kDppRowMirror>(x); x = x > y ? x : y;
  return x;
}

// max over the whole 64-lane wavefront; the result is wave-uniform
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  x = row16_max_u32(x);
  uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0);
  uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
  uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  a = a > b ? a : b;
  c = c > d ? c : d;
  return a > c ? a : c;
}

// Selection key: larger score wins, then the lower slot.  0 = "not evictable".
__device__ __forceinline__ uint32_t make_key(uint32_t score, uint32_t slot) {
  return ((score + 1u) << 20) | (0xFFFFFu - slot);
}
__device__ __forceinline__ int key_slot(uint32_t key) { return (int)(0xFFFFFu - (key & 0xFFFFFu)); }
// ---- a row of K, V or Q as the lanes hold it -----------------------------------------------
// A lane owns 8 consecutive head-dim elements of a row: HD/8 lanes per row, 64/(HD/8) rows per
// wave-wide load.  Eight consecutive elements as loaded (16 bytes of bf16 or 32 bytes of fp32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

template <bool BF16>
struct Raw8;
template <>
struct Raw8<true> {
  uint4 v;
  __device__ __forceinline__ void load(const void *p) { v = *(const uint4 *)p; }
  __device__ __forceinline__ void unpack(float (&x)[8]) const {
    x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
    x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
  }
};
template <>
struct Raw8<false> {
  float4 a, b;
  __device__ __forceinline__ void load(const void *p) {
    a = ((const float4 *)p)[0]; b = ((const float4 *)p)[1];
  }
  __device__ __forceinline__ void unpack(float (&x)[8]) const {
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
};

// q . k over the lane's eight elements.  bf16: four packed dot-products with fp32
// accumulation (products of bf16 values are exact in fp32); fp32: eight FMAs.
__device__ __forceinline__ float dot8(const Raw8<true> &q, const Raw8<true> &k) {
  float acc = 0.0f;
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, q.v.x),
                                        __builtin_bit_cast(bf16x2_t, k.v.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, q.v.y),
                                        __builtin_bit_cast(bf16x2_t, k.v.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, q.v.z),
                                        __builtin_bit_cast(bf16x2_t, k.v.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, q.v.w),
                                        __builtin_bit_cast(bf16x2_t, k.v.w), acc, false);
  return acc;
}
__device__ __forceinline__ float dot8(const Raw8<false> &q, const Raw8<false> &k) {
  float acc = q.a.x * k.a.x;
  acc = fmaf(q.a.y, k.a.y, acc); acc = fmaf(q.a.z, k.a.z, acc); acc = fmaf(q.a.w, k.a.w, acc);
  acc = fmaf(q.b.x, k.b.x, acc); acc = fmaf(q.b.y, k.b.y, acc); acc = fmaf(q.b.z, k.b.z, acc);
  acc = fmaf(q.b.w, k.b.w, acc);
  return acc;
}

// sum over the LPR adjacent lanes that share a row; the result is in every lane of the group
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f32<kDppQuadSwap1>(x);
  x += dpp_f32<kDppQuadSwap2>(x);
  if constexpr (LPR >= 8) x += dpp_f32<kDppRowHalfMirror>(x);
  if constexpr (LPR >= 16) x += dpp_f32<kDppRowMirror>(x);
  return x;
}

// L2-norm policy: bit pattern of the squared norm of a row whose 8-element pieces the HD/8
// lanes of a group hold -- eight products per lane in fp32, then a butterfly over the group.
// The same function serves the bulk kernel and the decode step, so a key gets the same word
// whichever entry point took its norm.  (fp32 summation of HD non-negative terms: within
// HD * 2^-24 relative of the exact value in any order.)
template <int HD, bool BF16>
__device__ __forceinline__ uint32_t norm2_bits_of_piece(const Raw8<BF16> &x) {
  return __float_as_uint(group_sum<HD / 8>(dot8(x, x)));
}

#endif  // __HIPCC__

}  // namespace lshe
