// lshe_decode_step: one time step of Algorithm 1 for every unit, as two or three kernels.
//
//   select_kernel   one workgroup per unit: hash the G queries and the new key (eq. 2),
//                   Hamming-score every occupied slot (eq. 5), pick the victim (eq. 6) with a
//                   DPP wave reduction + LDS across waves, overwrite the slot in place
//                   (Algorithm 1 steps 2-5).
//   attn_kernel     `splits` workgroups per unit stream disjoint slot ranges of the updated
//                   K/V cache once, each keeping an online-softmax state per query head
//                   (eq. 1); with more than one split a small combine_kernel merges the
//                   partial states.
//
// The victim is fully written before the attention kernel starts (kernel boundary), so
// readers of a head's codes or K/V never race with the in-place overwrite.
#include "lshe_hash_tile.h"
#include "lshe_kernels.h"

namespace lshe {

struct DecodeArgs {
  const void *R_dev, *q, *k_new, *v_new;
  const int32_t *pos;
  void *K, *V;
  uint32_t *code;
  int32_t *slot_pos, *n_valid;
  void *out;
  int32_t *evicted, *scores_dbg;
  uint32_t *codes_dbg;
  float *partials;
  int C, G, r, units_per_seq, n_sink, n_recent, S;
  float qscale;  // log2(e) / sqrt(d)
};

// ---- select: hash, score, argmax, overwrite ------------------------------------------------
template <int HD, int W, bool BF16>
__global__ __launch_bounds__(256) void select_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  const int u = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int C = a.C, G = a.G;

  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];  // G query codes, then the key code
  __shared__ uint32_t s_best[4];

  if (wave == 0) {
    RFrag<HD, W, BF16> rf;
    rf.load(a.R_dev, lane);
    const int row = lane & 31;
    const char *rowp = nullptr;
    if (row < G) rowp = (const char *)a.q + ((size_t)u * G + row) * HD * ES;
    else if (row == G) rowp = (const char *)a.k_new + (size_t)u * HD * ES;
    uint32_t code[W];
    hash_tile32<HD, W, BF16>(rowp, rf, a.r, lane, code);
    if (lane <= G) {
#pragma unroll
      for (int w = 0; w < W; ++w) {
        s_code[lane * W + w] = code[w];
        if (a.codes_dbg) a.codes_dbg[((size_t)u * (G + 1) + lane) * W + w] = code[w];
      }
    }
  }
  const int nv = a.n_valid[u];
  const int t = a.pos[u / a.units_per_seq];
  __syncthreads();

  const uint32_t *codes = a.code + (size_t)u * C * W;
  const int32_t *spos = a.slot_pos + (size_t)u * C;
  const bool masked = (a.n_sink | a.n_recent) != 0;
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t best = 0;
  for (int s = tid; s < nv; s += 256) {
    uint32_t sc = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) {
      const uint32_t c = codes[(size_t)s * W + w];
      for (int g = 0; g < G; ++g) sc += __popc(c ^ s_code[g * W + w]);
    }
    if (a.scores_dbg) a.scores_dbg[(size_t)u * C + s] = (int32_t)sc;
    bool ok = true;
    if (masked) {
      const int p = spos[s];
      ok = p >= a.n_sink && p <= newest_evictable;
    }
    const uint32_t key = ok ? make_key(sc, (uint32_t)s) : 0u;
    best = best > key ? best : key;
  }
  if (a.scores_dbg)
    for (int s = nv + tid; s < C; s += 256) a.scores_dbg[(size_t)u * C + s] = -1;

  best = wave_max_u32(best);
  if (lane == 0) s_best[wave] = best;
  __syncthreads();
  {
    const uint32_t b0 = s_best[0], b1 = s_best[1], b2 = s_best[2], b3 = s_best[3];
    const uint32_t m01 = b0 > b1 ? b0 : b1, m23 = b2 > b3 ? b2 : b3;
    best = m01 > m23 ? m01 : m23;
  }
  int e;
  if (nv < C) e = nv;                   // cache not full: append, nobody is evicted
  else if (best != 0u) e = key_slot(best);
  else e = -1;                          // inconsistent state (no evictable slot): leave the cache alone

  if (e >= 0) {
    constexpr int VEC = HD * ES / 16;   // 16-byte pieces per row
    if (tid < VEC) {
      ((uint4 *)((char *)a.K + ((size_t)u * C + e) * HD * ES))[tid] =
          ((const uint4 *)((const char *)a.k_new + (size_t)u * HD * ES))[tid];
    } else if (tid >= 64 && tid < 64 + VEC) {
      ((uint4 *)((char *)a.V + ((size_t)u * C + e) * HD * ES))[tid - 64] =
          ((const uint4 *)((const char *)a.v_new + (size_t)u * HD * ES))[tid - 64];
    } else if (tid >= 128 && tid < 128 + W) {
      a.code[((size_t)u * C + e) * W + (tid - 128)] = s_code[G * W + (tid - 128)];
    } else if (tid == 192) {
      a.slot_pos[(size_t)u * C + e] = t;
      if (nv < C) a.n_valid[u] = nv + 1;
    }
  }
  if (tid == 193 && a.evicted) a.evicted[u] = e;
}

// ---- attention over the updated cache ------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ void load8(const void *p, float (&x)[8]) {
  if constexpr (BF16) {
    const uint4 v = *(const uint4 *)p;
    x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
    x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
  } else {
    const float4 a = ((const float4 *)p)[0], b = ((const float4 *)p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

// Eight consecutive elements of a row as loaded (16 bytes of bf16 or 32 bytes of fp32).
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

template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f32<kDppQuadSwap1>(x);
  x += dpp_f32<kDppQuadSwap2>(x);
  if constexpr (LPR >= 8) x += dpp_f32<kDppRowHalfMirror>(x);
  if constexpr (LPR >= 16) x += dpp_f32<kDppRowMirror>(x);
  return x;
}

constexpr float kNegBig = -1.0e30f;

template <bool BF16>
__device__ __forceinline__ void store_out(void *out, size_t idx, float v) {
  if constexpr (BF16) ((uint16_t *)out)[idx] = (uint16_t)f32_to_bf16_bits(v);
  else ((float *)out)[idx] = v;
}

// A lane owns 8 consecutive head-dim elements of one row: LPR = HD/8 lanes per row and
// RPW = 64/LPR rows per wave-wide load, so every load instruction reads RPW whole rows
// (contiguous memory).  The four waves of a workgroup interleave at that granularity.
template <int HD, int G, bool BF16>
__global__ __launch_bounds__(kAttnThreads) void attn_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int LPR = HD / 8;
  constexpr int RPW = 64 / LPR;
  constexpr int NW = kAttnThreads / 64;
  constexpr int NS = NW * RPW;   // independent online-softmax streams per workgroup
  constexpr int U = BF16 ? 4 : 2;   // rows per lane per block (two blocks in flight)
  const int S = a.S;
  const int u = blockIdx.x / S, split = blockIdx.x - u * S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPR, rg = lane / LPR;
  const int nv = a.n_valid[u];

  int rps = (nv + S - 1) / S;
  rps = (rps + NS - 1) / NS * NS;
  const int r0 = split * rps;
  const int r1 = min(nv, r0 + rps);

  float q[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load8<BF16>((const char *)a.q + (((size_t)u * G + g) * HD + c * 8) * ES, q[g]);
#pragma unroll
    for (int i = 0; i < 8; ++i) q[g][i] *= a.qscale;
  }
  float m[G], l[G], o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig; l[g] = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[g][i] = 0.0f;
  }

  const char *Kb = (const char *)a.K + ((size_t)u * a.C * HD + c * 8) * ES;
  const char *Vb = (const char *)a.V + ((size_t)u * a.C * HD + c * 8) * ES;
  const int n_iter = r1 > r0 ? (r1 - r0 + U * NS - 1) / (U * NS) : 0;

  // Loads are unconditional (rows past the range re-read row r0 and are masked in the
  // arithmetic), so all of a block's loads are in flight together, and the next block is
  // requested before the current one is consumed.
  Raw8<BF16> kn[U], vn[U];
  auto request = [&](int it) {
#pragma unroll
    for (int j = 0; j < U; ++j) {
      int row = r0 + ((it * U + j) * NW + wave) * RPW + rg;
      row = row < r1 ? row : r0;
      kn[j].load(Kb + (size_t)row * HD * ES);
      vn[j].load(Vb + (size_t)row * HD * ES);
    }
  };
  if (n_iter > 0) request(0);
  for (int it = 0; it < n_iter; ++it) {
    Raw8<BF16> kc[U], vc[U];
    bool ok[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      kc[j] = kn[j]; vc[j] = vn[j];
      ok[j] = r0 + ((it * U + j) * NW + wave) * RPW + rg < r1;
    }
    if (it + 1 < n_iter) request(it + 1);

    float s[U][G];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      float kf[8];
      kc[j].unpack(kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(q[g][i], kf[i], acc);
        s[j][g] = group_sum<LPR>(acc);
      }
    }
    float p[U][G], corr[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int j = 0; j < U; ++j) mn = ok[j] ? fmaxf(mn, s[j][g]) : mn;
      corr[g] = __builtin_amdgcn_exp2f(m[g] - mn);
      m[g] = mn;
      float ps = 0.0f;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        p[j][g] = ok[j] ? __builtin_amdgcn_exp2f(s[j][g] - mn) : 0.0f;
        ps += p[j][g];
      }
      l[g] = fmaf(l[g], corr[g], ps);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[g][i] *= corr[g];
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      float vf[8];
      vc[j].unpack(vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] = fmaf(p[j][g], vf[i], o[g][i]);
    }
  }

  // ---- merge the NS streams of the workgroup through LDS ----------------------------------
  __shared__ float sm_m[NS][G], sm_l[NS][G];
  __shared__ __align__(16) float sm_o[NS][HD];
  const int stream = wave * RPW + rg;
  if (c == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) { sm_m[stream][g] = m[g]; sm_l[stream][g] = l[g]; }
  }
  float *part = a.partials + ((size_t)u * S + split) * G * (HD + 2);
#pragma unroll
  for (int g = 0; g < G; ++g) {
    __syncthreads();   // previous round's readers are done (and sm_m/sm_l are visible)
    *(float4 *)&sm_o[stream][c * 8] = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
    *(float4 *)&sm_o[stream][c * 8 + 4] = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
    __syncthreads();
    if (tid < HD) {
      float M = kNegBig;
#pragma unroll
      for (int k = 0; k < NS; ++k) M = fmaxf(M, sm_m[k][g]);
      float O = 0.0f, Lsum = 0.0f;
#pragma unroll
      for (int k = 0; k < NS; ++k) {
        const float w = __builtin_amdgcn_exp2f(sm_m[k][g] - M);
        O = fmaf(w, sm_o[k][tid], O);
        Lsum = fmaf(w, sm_l[k][g], Lsum);
      }
      if (S == 1) {
        store_out<BF16>(a.out, ((size_t)u * G + g) * HD + tid, Lsum > 0.0f ? O / Lsum : 0.0f);
      } else {
        part[g * (HD + 2) + 2 + tid] = O;
        if (tid == 0) { part[g * (HD + 2)] = M; part[g * (HD + 2) + 1] = Lsum; }
      }
    }
  }
}

// Merge the S partial softmax states of every unit (only launched when S > 1).  A separate
// launch rather than "last workgroup to finish merges": the kernel boundary makes the
// partials visible across the chip's L2 slices, whereas device-scope fences inside the
// streaming kernel write back and invalidate a whole L2 per workgroup and cost ten times
// the kernel itself.
template <int HD, int G, bool BF16>
__global__ __launch_bounds__(HD) void combine_kernel(const DecodeArgs a) {
  const int u = blockIdx.x, tid = threadIdx.x, S = a.S;
  const float *pu = a.partials + (size_t)u * S * G * (HD + 2);
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float M = kNegBig;
    for (int k = 0; k < S; ++k) M = fmaxf(M, pu[((size_t)k * G + g) * (HD + 2)]);
    float O = 0.0f, Lsum = 0.0f;
    for (int k = 0; k < S; ++k) {
      const float *pk = pu + ((size_t)k * G + g) * (HD + 2);
      const float w = __builtin_amdgcn_exp2f(pk[0] - M);
      O = fmaf(w, pk[2 + tid], O);
      Lsum = fmaf(w, pk[1], Lsum);
    }
    store_out<BF16>(a.out, ((size_t)u * G + g) * HD + tid, Lsum > 0.0f ? O / Lsum : 0.0f);
  }
}

template <int HD, bool BF16>
static int launch_select(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const unsigned units = (unsigned)m.units;
  if (m.W == 1)
    hipLaunchKernelGGL((select_kernel<HD, 1, BF16>), dim3(units), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((select_kernel<HD, 2, BF16>), dim3(units), dim3(256), 0, st, a);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

template <int HD, bool BF16>
static int launch_attend(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const dim3 grid((unsigned)m.units * (unsigned)a.S), block(kAttnThreads);
  switch (m.G) {
    case 1: hipLaunchKernelGGL((attn_kernel<HD, 1, BF16>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((attn_kernel<HD, 2, BF16>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((attn_kernel<HD, 4, BF16>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((attn_kernel<HD, 8, BF16>), grid, block, 0, st, a); break;
    default: return LSHE_UNSUPPORTED;
  }
  LSHE_HIP_TRY(hipGetLastError());
  if (a.S > 1) {
    const dim3 cgrid((unsigned)m.units), cblock(HD);
    switch (m.G) {
      case 1: hipLaunchKernelGGL((combine_kernel<HD, 1, BF16>), cgrid, cblock, 0, st, a); break;
      case 2: hipLaunchKernelGGL((combine_kernel<HD, 2, BF16>), cgrid, cblock, 0, st, a); break;
      case 4: hipLaunchKernelGGL((combine_kernel<HD, 4, BF16>), cgrid, cblock, 0, st, a); break;
      default: hipLaunchKernelGGL((combine_kernel<HD, 8, BF16>), cgrid, cblock, 0, st, a); break;
    }
    LSHE_HIP_TRY(hipGetLastError());
  }
  return LSHE_OK;
}

enum { kPhaseSelect = 1, kPhaseAttend = 2 };

static int run_phases(const Dims &m, const DecodeArgs &a, int phases, hipStream_t st) {
  const bool bf = m.dtype == LSHE_BF16;
  int rc = LSHE_OK;
  if (phases & kPhaseSelect) {
    if (m.d == 128) rc = bf ? launch_select<128, true>(m, a, st) : launch_select<128, false>(m, a, st);
    else if (m.d == 64) rc = bf ? launch_select<64, true>(m, a, st) : launch_select<64, false>(m, a, st);
    else rc = LSHE_UNSUPPORTED;
    if (rc != LSHE_OK) return rc;
  }
  if (phases & kPhaseAttend) {
    if (m.d == 128) rc = bf ? launch_attend<128, true>(m, a, st) : launch_attend<128, false>(m, a, st);
    else if (m.d == 64) rc = bf ? launch_attend<64, true>(m, a, st) : launch_attend<64, false>(m, a, st);
    else rc = LSHE_UNSUPPORTED;
  }
  return rc;
}

// Argument checks and DecodeArgs shared by the three entry points; pointers a phase does not
// use may be NULL for that phase.
static int decode_common(const lshe_config *cfg, const void *R_dev, const void *q_new,
                         const void *k_new, const void *v_new, const int32_t *pos, void *K_cache,
                         void *V_cache, uint32_t *code_cache, int32_t *slot_pos, int32_t *n_valid,
                         void *out, int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                         void *workspace, size_t workspace_bytes, void *stream, int phases) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (!q_new || !K_cache || !V_cache || !n_valid || !workspace) return LSHE_INVALID_ARG;
  if ((phases & kPhaseSelect) &&
      (!R_dev || !k_new || !v_new || !pos || !code_cache || !slot_pos))
    return LSHE_INVALID_ARG;
  if ((phases & kPhaseAttend) && !out) return LSHE_INVALID_ARG;
  const Dims m = dims_of(cfg);
  if (m.G != 1 && m.G != 2 && m.G != 4 && m.G != 8) return LSHE_UNSUPPORTED;
  if (workspace_bytes < decode_ws_bytes(m)) return LSHE_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)workspace & 255u) != 0) return LSHE_INVALID_ARG;

  DecodeArgs a;
  a.R_dev = R_dev; a.q = q_new; a.k_new = k_new; a.v_new = v_new; a.pos = pos;
  a.K = K_cache; a.V = V_cache; a.code = code_cache; a.slot_pos = slot_pos; a.n_valid = n_valid;
  a.out = out; a.evicted = evicted; a.scores_dbg = scores_dbg; a.codes_dbg = codes_dbg;
  a.partials = (float *)workspace;
  a.C = m.C; a.G = m.G; a.r = m.r; a.units_per_seq = m.L * m.H;
  a.n_sink = m.n_sink; a.n_recent = m.n_recent;
  a.S = attn_splits(m.units, m.C);
  a.qscale = (float)(1.4426950408889634 / sqrt((double)m.d));
  return run_phases(m, a, phases, (hipStream_t)stream);
}

}  // namespace lshe

using namespace lshe;

extern "C" int lshe_decode_step(const lshe_config *cfg, const void *R_dev, const void *q_new,
                                const void *k_new, const void *v_new, const int32_t *pos,
                                void *K_cache, void *V_cache, uint32_t *code_cache,
                                int32_t *slot_pos, int32_t *n_valid, void *out, int32_t *evicted,
                                int32_t *scores_dbg, uint32_t *codes_dbg, void *workspace,
                                size_t workspace_bytes, void *stream) {
  return decode_common(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                       n_valid, out, evicted, scores_dbg, codes_dbg, workspace, workspace_bytes,
                       stream, kPhaseSelect | kPhaseAttend);
}

extern "C" int lshe_decode_select(const lshe_config *cfg, const void *R_dev, const void *q_new,
                                  const void *k_new, const void *v_new, const int32_t *pos,
                                  void *K_cache, void *V_cache, uint32_t *code_cache,
                                  int32_t *slot_pos, int32_t *n_valid, int32_t *evicted,
                                  int32_t *scores_dbg, uint32_t *codes_dbg, void *workspace,
                                  size_t workspace_bytes, void *stream) {
  return decode_common(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                       n_valid, nullptr, evicted, scores_dbg, codes_dbg, workspace, workspace_bytes,
                       stream, kPhaseSelect);
}

extern "C" int lshe_decode_attend(const lshe_config *cfg, const void *q_new, const void *K_cache,
                                  const void *V_cache, const int32_t *n_valid, void *out,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  return decode_common(cfg, nullptr, q_new, nullptr, nullptr, nullptr, (void *)K_cache,
                       (void *)V_cache, nullptr, nullptr, (int32_t *)n_valid, out, nullptr, nullptr,
                       nullptr, workspace, workspace_bytes, stream, kPhaseAttend);
}
