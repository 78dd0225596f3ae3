// Sign-random-projection of a 32-row tile on the matrix cores (Section 2, eq. (2)).
//
// One wavefront hashes 32 vectors at a time: P^T[32 bits][32 rows] = R[32][d] * X^T[d][32]
// per code word with v_mfma_f32_32x32x{16 bf16, 2 f32}.  With R as the first operand the
// accumulator layout puts ONE input row (column j = lane % 32) in every lane and hash bits
// i = 8*(v/4) + 4*(lane/32) + v%4 in accumulator registers v = 0..15, so a lane packs 16 of
// its row's bits from the accumulators' sign bits with one v_alignbit each, and a single
// exchange with lane ^ 32 completes the 32-bit word.  No LDS, no per-bit compares.
//
// Bit = 1 iff the projection is >= 0.  The accumulators start at +0.0, so an exactly-zero
// projection comes out as +0.0 (sign bit clear) and signs to 1 as the definition requires.
//
// Both the bulk hashing kernel and the decode-step kernel call hash_tile32, so a vector
// gets the same code whichever entry point hashed it.
#pragma once

#include "lshe_common.h"

namespace lshe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// The d-index each lane supplies per MFMA k-step is the same for the X and the R operand,
// so any fixed assignment gives the exact contraction over d:
//   bf16: k-step kk (HD/16 of them), half = lane/32, element i (0..7): d = 16*kk + 8*half + i
//   f32 : load j (HD/8 of them), half, element i (0..3) -> one k-step each: d = 8*j + 4*half + i

template <int HD, int W, bool BF16>
struct RFrag;

template <int HD, int W>
struct RFrag<HD, W, true> {
  static constexpr bool kResident = true;
  bf16x8_t b[W][HD / 16];
  __device__ __forceinline__ bf16x8_t get(int w, int kk) const { return b[w][kk]; }
  __device__ __forceinline__ void load(const void *R_dev, int lane) {
    const uint16_t *R = (const uint16_t *)R_dev;
    const int n = lane & 31, half = lane >> 5;
#pragma unroll
    for (int w = 0; w < W; ++w)
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk)
        b[w][kk] = *(const bf16x8_t *)(R + (size_t)(32 * w + n) * HD + 16 * kk + 8 * half);
  }
};

template <int HD, int W>
struct RFrag<HD, W, false> {
  static constexpr bool kResident = false;
  const float *R;
  __device__ __forceinline__ void load(const void *R_dev, int) { R = (const float *)R_dev; }
};

// Turn one accumulator tile into the code word of row (lane % 32); valid in every lane.
__device__ __forceinline__ uint32_t sign_pack32(const f32x16_t &acc, int half) {
  uint32_t sg = 0;
#pragma unroll
  for (int v = 15; v >= 0; --v)   // sg = (sg << 1) | signbit(acc[v])
    sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(acc[v]), 31);
  sg = ~sg & 0xFFFFu;             // bit v = (acc[v] >= 0)
  // accumulator v holds hash bit 8*(v/4) + v%4 (+4 in the upper half-wave): spread the nibbles
  uint32_t t = (sg & 0x000Fu) | ((sg & 0x00F0u) << 4) | ((sg & 0x0F00u) << 8) | ((sg & 0xF000u) << 12);
  t <<= 4 * half;
  return t | (uint32_t)__shfl_xor((int)t, 32);
}

// A lane's share of one 32-row tile of X: the elements of row (lane % 32) that the lane feeds
// to the MFMAs.  load() issues every request before anything waits, so a tile costs one
// memory round trip and the next tile can be requested while the current one is multiplied.
// rowp must be readable in every lane: a lane whose row is padding passes any valid row and
// ignores the code it gets (an input row only influences its own column of the product).
template <int HD, bool BF16>
struct XFrag;

template <int HD>
struct XFrag<HD, true> {
  bf16x8_t a[HD / 16];
  __device__ __forceinline__ void load(const void *rowp, int lane) {
    const uint16_t *x = (const uint16_t *)rowp + 8 * (lane >> 5);
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) a[kk] = *(const bf16x8_t *)(x + 16 * kk);
  }
};

template <int HD>
struct XFrag<HD, false> {
  f32x4_t a[HD / 8];
  __device__ __forceinline__ void load(const void *rowp, int lane) {
    const float *x = (const float *)rowp + 4 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < HD / 8; ++j) a[j] = *(const f32x4_t *)(x + 8 * j);
  }
};

// On return code[w] holds word w of row (lane % 32) in every lane; bits >= r are cleared.
template <int HD, int W, bool BF16, typename RF>
__device__ __forceinline__ void hash_tile32(const XFrag<HD, BF16> &x, const RF &rf, int r, int lane,
                                            uint32_t (&code)[W]) {
  const int half = lane >> 5;
  if constexpr (BF16) {
    static_assert(RF::kResident, "bf16 hashing keeps R in registers");
#pragma unroll
    for (int w = 0; w < W; ++w) {
      f32x16_t acc = (f32x16_t)(0.0f);
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rf.get(w, kk), x.a[kk], acc, 0, 0, 0);
      code[w] = sign_pack32(acc, half);
    }
  } else {
    const int n = lane & 31;
    f32x16_t acc[W];
#pragma unroll
    for (int w = 0; w < W; ++w) acc[w] = (f32x16_t)(0.0f);
#pragma unroll
    for (int j = 0; j < HD / 8; ++j) {
#pragma unroll
      for (int w = 0; w < W; ++w) {
        const f32x4_t b = *(const f32x4_t *)(rf.R + (size_t)(32 * w + n) * HD + 8 * j + 4 * half);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[w] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[i], x.a[j][i], acc[w], 0, 0, 0);
      }
    }
#pragma unroll
    for (int w = 0; w < W; ++w) code[w] = sign_pack32(acc[w], half);
  }
  // rows of R beyond r are zero, so their projections are 0 and sign to 1: clear those bits
  const int tail = r - 32 * (W - 1);
  if (tail < 32) code[W - 1] &= (1u << tail) - 1u;
}

}  // namespace lshe
