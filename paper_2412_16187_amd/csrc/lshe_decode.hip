// lshe_decode_step: one time step of Algorithm 1 for every unit.
//
// Launch plans, chosen on the host from the number of units and the budget (lshe_decode_plan
// names them):
//
//   fused, one-wave select (128..1023 units, code table of 1024..4096 words per unit)
//       ONE kernel, one workgroup of 8 waves per unit.  Wave 0 hashes the G queries and the
//       new key (eq. 2), Hamming-scores every occupied slot (eq. 5), picks the victim (eq. 6)
//       and overwrites the slot in place (Algorithm 1 steps 2-5) on its own, while the other
//       waves already stream the unit's K/V with an online softmax per query head (eq. 1);
//       they pick the victim's slot up from LDS when it appears and stream again the few
//       chunks that held the victim's old row.
//
//   fused, all waves select (other cases with >= 128 units, or budgets <= 512)
//       ONE kernel: every wave requests its first K/V rows, the workgroup selects together
//       (DPP wave reduction + LDS across waves), then streams.
//
//   split (few units)   attn_local_kernel (`splits` workgroups per unit over disjoint slot
//       ranges, each selecting over its own range and setting its candidate row aside) ->
//       merge_local_kernel (victim = best candidate of the unit, merge of the partial softmax
//       states, Algorithm 1's overwrite).  The kernel boundary makes the candidates and the
//       partial states visible chip-wide; device-scope fences inside the streaming kernel were
//       measured at ten times its cost.  The stage-wise calls (lshe_decode_select,
//       lshe_decode_attend) run select_kernel (one workgroup per unit), then attn_kernel ->
//       combine_kernel.
//
//   groups of 8 query heads (budgets above 512)   select_kernel -> attn_kernel with two
//       workgroups per unit and slot range, 4 heads each (-> combine_kernel if there are ranges).
//
// In the single-kernel and two-launch plans the victim's row is never taken from memory by the
// attention: the lanes put the new key/value in its place from registers, so it does not
// matter what memory holds while the slot is being overwritten.
#include <atomic>
#include <mutex>

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
  float *evicted_mass;   // nullable out [units][G]
  float *victim_logit;   // workspace [units][G]: scaled logit of the victim's old key per head
  float *partials;
  int32_t *sel_out;      // workspace [units][4]: occupied slots before the step, token index, key code words (see attn_local_kernel)
  int32_t *status;       // workspace status word: kernels OR LSHE_STATUS_* bits into it
  int spin_limit;        // polls of the victim word before a streaming wave gives up (one-wave select)
  int withhold_victim;   // test hook: the select wave does not publish the slot
  int C, G, r, units_per_seq, n_sink, n_recent, S, policy;
  float qscale;  // log2(e) / sqrt(d)
};


// ============================================================================================
// select: hash, score, argmax (Algorithm 1 step 1)
// ============================================================================================

// One wave hashes rows 0..G-1 = queries, row G = new key; result in s_code[(G+1)*W].
// issue() requests R and the rows whole (one memory round trip on the step's critical path;
// the registers are free this early in the kernel); finish() multiplies and stores the codes.
// Lanes past row G hash the key again and drop the result.
template <int HD, int W, bool BF16>
struct StepHash {
  XFrag<HD, BF16> x;
  RFrag<HD, W, BF16> rf;
  Raw8<BF16> kn;   // L2-norm policy: the lane's piece of the new key

  __device__ __forceinline__ void issue(const DecodeArgs &a, int u, int lane) {
    constexpr int ES = BF16 ? 2 : 4;
    if (a.policy == LSHE_POLICY_L2NORM) {   // no projection: the first HD/8 lanes take the key
      kn.load((const char *)a.k_new + ((size_t)u * HD + (lane % (HD / 8)) * 8) * ES);
      return;
    }
    const int row = lane & 31;
    const char *rowp = row < a.G ? (const char *)a.q + ((size_t)u * a.G + row) * HD * ES
                                 : (const char *)a.k_new + (size_t)u * HD * ES;
    x.load(rowp, lane);
    rf.load(a.R_dev, lane);
  }

  __device__ __forceinline__ void finish(const DecodeArgs &a, int u, int lane, uint32_t *s_code) {
    constexpr int ES = BF16 ? 2 : 4;
    const int G = a.G;
    if (a.policy == LSHE_POLICY_L2NORM) {
      // the key's code is the bit pattern of its squared norm (every group of HD/8 lanes holds
      // the whole key, so every lane ends up with the word); queries have no code
      const uint32_t nb = norm2_bits_of_piece<HD, BF16>(kn);
      if (lane <= G) {
        const uint32_t c = lane == G ? nb : 0u;
        s_code[lane * W] = c;
        if (a.codes_dbg) a.codes_dbg[((size_t)u * (G + 1) + lane) * W] = c;
      }
      return;
    }
    uint32_t code[W];
    hash_tile32<HD, W, BF16>(x, rf, a.r, lane, code);
    if (lane <= G) {
#pragma unroll
      for (int w = 0; w < W; ++w) {
        s_code[lane * W + w] = code[w];
        if (a.codes_dbg) a.codes_dbg[((size_t)u * (G + 1) + lane) * W + w] = code[w];
      }
    }
  }
};

template <int HD, int W, bool BF16>
__device__ __forceinline__ void hash_step_inputs(const DecodeArgs &a, int u, int lane,
                                                 uint32_t *s_code) {
  StepHash<HD, W, BF16> h;
  h.issue(a, u, lane);
  h.finish(a, u, lane, s_code);
}

// The first kScorePrefetch slots of each thread's share of the code table (and their token
// positions when some tokens are protected), requested early so that scoring does not
// start with a round trip to memory.
constexpr int kScorePrefetch = 4;
constexpr int kScoreBatch = 8;   // slots per thread requested together beyond the prefetched ones
constexpr int kSelectSmallBudget = 2048;   // select_kernel: 256 threads up to here, 1024 beyond

template <int W, int NT>
struct CodePrefetch {
  uint32_t c[kScorePrefetch][W];
  int p[kScorePrefetch];
  __device__ __forceinline__ void load(const DecodeArgs &a, int u, int tid) {
    const uint32_t *codes = a.code + (size_t)u * a.C * W;
    const int32_t *spos = a.slot_pos + (size_t)u * a.C;
    const bool masked = (a.n_sink | a.n_recent) != 0;
#pragma unroll
    for (int k = 0; k < kScorePrefetch; ++k) {
      int s = tid + k * NT;
      s = s < a.C ? s : 0;   // any slot of the unit is a valid address; validity is checked later
#pragma unroll
      for (int w = 0; w < W; ++w) c[k][w] = codes[(size_t)s * W + w];
      p[k] = masked ? spos[s] : 0;
    }
  }
};

// score_and_select's scan in the common case -- no protected tokens, no debug output -- with the
// group size known at compile time and the step's query codes in registers: the thread's best
// key (0: none).
template <int W, int NT, int GT>
__device__ __forceinline__ uint32_t score_scan_plain(const DecodeArgs &a, int u, int nv, int tid,
                                                     const CodePrefetch<W, NT> &pre, const uint32_t *s_code) {
  const uint32_t *codes = a.code + (size_t)u * a.C * W;
  uint32_t qc[GT][W];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int w = 0; w < W; ++w) qc[g][w] = s_code[g * W + w];
  uint32_t best = 0;
  auto visit = [&](int s, const uint32_t (&c)[W]) __attribute__((always_inline)) {
    uint32_t sc = 0;
#pragma unroll
    for (int w = 0; w < W; ++w)
#pragma unroll
      for (int g = 0; g < GT; ++g) sc += __popc(c[w] ^ qc[g][w]);
    const uint32_t key = s < nv ? make_key(sc, (uint32_t)s) : 0u;
    best = best > key ? best : key;
  };
#pragma unroll
  for (int k = 0; k < kScorePrefetch; ++k) visit(tid + k * NT, pre.c[k]);
  for (int s0 = tid + kScorePrefetch * NT; s0 < nv; s0 += kScoreBatch * NT) {
    uint32_t c[kScoreBatch][W];
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) {
      const int s = s0 + b * NT;
      const int sl = s < nv ? s : 0;   // slot 0 stands in past the end; its key is dropped
#pragma unroll
      for (int w = 0; w < W; ++w) c[b][w] = codes[(size_t)sl * W + w];
    }
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) visit(s0 + b * NT, c[b]);
  }
  return best;
}

// Every thread of the workgroup calls this after s_code is visible.  Returns the slot to
// write: n_valid while the cache is filling, else the evictable slot with the largest summed
// Hamming distance (lowest slot on ties); -1 if no slot is evictable (inconsistent state).
// (PLAIN_PATH: also compile the compact scan of the common case; the stage-wise select kernel
// gains 10-30 % from it, the single-kernel step nothing, and its smallest shapes lose 1-2 %
// to the extra code)
template <int W, int NT, bool PLAIN_PATH = false>
__device__ __forceinline__ int score_and_select(const DecodeArgs &a, int u, int nv, int t, int tid,
                                                const CodePrefetch<W, NT> &pre,
                                                const uint32_t *s_code, uint32_t *s_best) {
  constexpr int NWAVES = NT / 64;
  const int C = a.C, G = a.G, lane = tid & 63, wave = tid >> 6;
  const uint32_t *codes = a.code + (size_t)u * C * W;
  const int32_t *spos = a.slot_pos + (size_t)u * C;
  const bool masked = (a.n_sink | a.n_recent) != 0;
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t best = 0;
  auto visit = [&](int s, const uint32_t (&c)[W], int p) __attribute__((always_inline)) {
    uint32_t sc = 0;
#pragma unroll
    for (int w = 0; w < W; ++w)
      for (int g = 0; g < G; ++g) sc += __popc(c[w] ^ s_code[g * W + w]);
    if (a.scores_dbg) a.scores_dbg[(size_t)u * C + s] = (int32_t)sc;
    const bool ok = !masked || (p >= a.n_sink && p <= newest_evictable);
    const uint32_t key = ok ? make_key(sc, (uint32_t)s) : 0u;
    best = best > key ? best : key;
  };
  const bool plain = PLAIN_PATH && !masked && a.scores_dbg == nullptr;
  if (plain) {
    switch (G) {
      case 1: best = score_scan_plain<W, NT, 1>(a, u, nv, tid, pre, s_code); break;
      case 2: best = score_scan_plain<W, NT, 2>(a, u, nv, tid, pre, s_code); break;
      case 4: best = score_scan_plain<W, NT, 4>(a, u, nv, tid, pre, s_code); break;
      default: best = score_scan_plain<W, NT, 8>(a, u, nv, tid, pre, s_code); break;
    }
  }
#pragma unroll
  for (int k = 0; k < kScorePrefetch; ++k) {
    const int s = tid + k * NT;
    if (!plain && s < nv) visit(s, pre.c[k], pre.p[k]);
  }
  // the rest of the table in batches: kScoreBatch independent requests per thread, then the
  // arithmetic (one request at a time would cost a memory round trip per slot)
  for (int s0 = tid + kScorePrefetch * NT; !plain && s0 < nv; s0 += kScoreBatch * NT) {
    uint32_t c[kScoreBatch][W];
    int p[kScoreBatch];
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) {
      const int s = s0 + b * NT;
      const int sl = s < nv ? s : 0;   // slot 0 stands in past the end; not visited
#pragma unroll
      for (int w = 0; w < W; ++w) c[b][w] = codes[(size_t)sl * W + w];
      p[b] = masked ? spos[sl] : 0;
    }
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) {
      const int s = s0 + b * NT;
      if (s < nv) visit(s, c[b], p[b]);
    }
  }
  if (a.scores_dbg)
    for (int s = nv + tid; s < C; s += NT) a.scores_dbg[(size_t)u * C + s] = -1;

  best = wave_max_u32(best);
  if (lane == 0) s_best[wave] = best;
  lds_barrier();   // also: every thread has finished reading the code table
#pragma unroll
  for (int k = 0; k < NWAVES; ++k) {
    const uint32_t o = s_best[k];
    best = best > o ? best : o;
  }
  if (nv < C) return nv;
  return best != 0u ? key_slot(best) : -1;
}

// Section 4.8's attention loss, per step: to report the attention probability that falls on
// the victim, its logit against every query head is taken from the key in slot e as it stands
// BEFORE the overwrite.  The first HD/8 lanes of the workgroup each take 8 elements; vl[g]
// receives q_g . k_e * log2(e)/sqrt(d), or a very negative number when nothing is evicted
// (cache still filling), which turns into a mass of zero.
template <int HD, bool BF16>
__device__ __forceinline__ void victim_logits(const DecodeArgs &a, int u, int e, bool evicting,
                                              int tid, float *vl);
// L2-norm policy: the evictable slot whose code word (bit pattern of the squared key norm) is
// largest, lowest slot on ties.  The 52-bit (norm, ~slot) key is reduced as two 32-bit maxima.
// s_best has room for 2 * NT/64 words.
template <int NT>
__device__ __forceinline__ int select_l2(const DecodeArgs &a, int u, int nv, int t, int tid,
                                         const CodePrefetch<1, NT> &pre, uint32_t *s_best) {
  constexpr int NWAVES = NT / 64;
  const int C = a.C, lane = tid & 63, wave = tid >> 6;
  const uint32_t *codes = a.code + (size_t)u * C;
  const int32_t *spos = a.slot_pos + (size_t)u * C;
  const bool masked = (a.n_sink | a.n_recent) != 0;
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t hi = 0, lo = 0;   // hi = norm bits + 1 (0 = nothing evictable), lo = 0xFFFFF - slot
  auto visit = [&](int s, uint32_t c, int p) __attribute__((always_inline)) {
    if (a.scores_dbg) a.scores_dbg[(size_t)u * C + s] = (int32_t)c;
    const bool ok = !masked || (p >= a.n_sink && p <= newest_evictable);
    const uint32_t h = ok ? c + 1u : 0u;
    if (h > hi) { hi = h; lo = 0xFFFFFu - (uint32_t)s; }   // slots come in ascending order
  };
#pragma unroll
  for (int k = 0; k < kScorePrefetch; ++k) {
    const int s = tid + k * NT;
    if (s < nv) visit(s, pre.c[k][0], pre.p[k]);
  }
  for (int s0 = tid + kScorePrefetch * NT; s0 < nv; s0 += kScoreBatch * NT) {
    uint32_t c[kScoreBatch];
    int p[kScoreBatch];
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) {
      const int s = s0 + b * NT;
      const int sl = s < nv ? s : 0;
      c[b] = codes[sl];
      p[b] = masked ? spos[sl] : 0;
    }
#pragma unroll
    for (int b = 0; b < kScoreBatch; ++b) {
      const int s = s0 + b * NT;
      if (s < nv) visit(s, c[b], p[b]);
    }
  }
  if (a.scores_dbg)
    for (int s = nv + tid; s < C; s += NT) a.scores_dbg[(size_t)u * C + s] = -1;

  const uint32_t whi = wave_max_u32(hi);
  const uint32_t wlo = wave_max_u32(hi == whi ? lo : 0u);
  if (lane == 0) { s_best[wave] = whi; s_best[NWAVES + wave] = wlo; }
  lds_barrier();   // also: every thread has finished reading the code table
  uint32_t bhi = 0, blo = 0;
#pragma unroll
  for (int k = 0; k < NWAVES; ++k) {
    const uint32_t h = s_best[k], l = s_best[NWAVES + k];
    if (h > bhi || (h == bhi && l > blo)) { bhi = h; blo = l; }
  }
  if (nv < C) return nv;
  return bhi != 0u ? (int)(0xFFFFFu - blo) : -1;
}

// Algorithm 1 steps 2-5: the new key, value, code and position replace slot e.
template <int HD, int W, bool BF16>
__device__ __forceinline__ void overwrite_slot(const DecodeArgs &a, int u, int e, int nv, int t,
                                               int tid, const uint32_t *s_code) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int VEC = HD * ES / 16;   // 16-byte pieces per row (<= 32)
  const int C = a.C;
  if (e >= 0) {
    if (tid < VEC) {
      ((uint4 *)((char *)a.K + ((size_t)u * C + e) * HD * ES))[tid] =
          ((const uint4 *)((const char *)a.k_new + (size_t)u * HD * ES))[tid];
    } else if (tid >= 64 && tid < 64 + VEC) {
      ((uint4 *)((char *)a.V + ((size_t)u * C + e) * HD * ES))[tid - 64] =
          ((const uint4 *)((const char *)a.v_new + (size_t)u * HD * ES))[tid - 64];
    } else if (tid >= 128 && tid < 128 + W) {
      a.code[((size_t)u * C + e) * W + (tid - 128)] = s_code[a.G * W + (tid - 128)];
    } else if (tid == 192) {
      a.slot_pos[(size_t)u * C + e] = t;
      if (nv < C) a.n_valid[u] = nv + 1;
    }
  }
  if (tid == 193 && a.evicted) a.evicted[u] = e;
}

// NT threads per unit: with few units the select is a chain of memory round trips, and a
// bigger workgroup has more of a long code table in flight per round trip.
template <int HD, int W, bool BF16, int NT>
__global__ __launch_bounds__(NT) void select_kernel(const DecodeArgs a) {
  const int u = blockIdx.x, tid = threadIdx.x;
  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];
  __shared__ uint32_t s_best[2 * NT / 64];
  const int nv = a.n_valid[u];
  const int t = a.pos[u / a.units_per_seq];
  CodePrefetch<W, NT> pre;
  pre.load(a, u, tid);
  if (tid < 64) hash_step_inputs<HD, W, BF16>(a, u, tid, s_code);
  lds_barrier();
  int e;
  if constexpr (W == 1) {
    e = a.policy == LSHE_POLICY_L2NORM ? select_l2<NT>(a, u, nv, t, tid, pre, s_best)
                                       : score_and_select<W, NT, true>(a, u, nv, t, tid, pre, s_code, s_best);
  } else {
    e = score_and_select<W, NT, true>(a, u, nv, t, tid, pre, s_code, s_best);
  }
  if (a.evicted_mass) {   // read the victim's key before it is overwritten
    victim_logits<HD, BF16>(a, u, e, nv == a.C && e >= 0, tid, a.victim_logit + (size_t)u * a.G);
    lds_barrier();
  }
  overwrite_slot<HD, W, BF16>(a, u, e, nv, t, tid, s_code);
}

// ============================================================================================
// attention over the updated cache (eq. 1)
// ============================================================================================

// Value of x held by lane (id ^ XOR); defined in the lanes whose id has that bit clear.
//   32: v_permlane32_swap exchanges the upper half of its first operand with the lower half
//       of its second, so with both operands = x the second result holds x[l+32] in lanes l < 32;
//   16: v_permlane16_swap does the same with odd and even rows of 16 lanes;
//    8: DPP rotate by 8 inside a row of 16.
template <int XOR>
__device__ __forceinline__ float lane_xor(float x) {
  typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
  const unsigned v = __float_as_uint(x);
  if constexpr (XOR == 32) {
    const u32x2_t r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return __uint_as_float(r.y);
  } else if constexpr (XOR == 16) {
    const u32x2_t r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return __uint_as_float(r.y);
  } else {
    static_assert(XOR == 8, "unsupported lane distance");
    return dpp_f32<0x128>(x);   // row_ror:8
  }
}

constexpr float kNegBig = -1.0e30f;

template <int HD, bool BF16>
__device__ __forceinline__ void victim_logits(const DecodeArgs &a, int u, int e, bool evicting,
                                              int tid, float *vl) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int LPR = HD / 8;
  if (tid >= LPR) return;
  if (!evicting) {
    if (tid < a.G) vl[tid] = kNegBig;
    return;
  }
  Raw8<BF16> k;
  k.load((const char *)a.K + (((size_t)u * a.C + e) * HD + tid * 8) * ES);
  for (int g = 0; g < a.G; ++g) {
    Raw8<BF16> q;
    q.load((const char *)a.q + (((size_t)u * a.G + g) * HD + tid * 8) * ES);
    const float x = group_sum<LPR>(dot8(q, k)) * a.qscale;
    if (tid == 0) vl[g] = x;
  }
}

template <bool BF16>
__device__ __forceinline__ void store_out(void *out, size_t idx, float v) {
  if constexpr (BF16) ((uint16_t *)out)[idx] = (uint16_t)f32_to_bf16_bits(v);
  else ((float *)out)[idx] = v;
}

// One workgroup's share of a unit's attention.  A lane owns 8 consecutive head-dim elements
// of one row: LPR = HD/8 lanes per row and RPW = 64/LPR rows per wave-wide load, so every
// load instruction reads RPW whole rows (contiguous memory).  The unit of work is a chunk of
// CH = U*RPW consecutive rows (U = 2 loads of K and of V per lane).  Each (wave, row-group)
// pair runs its own online softmax over the chunks its wave takes.
//
// Which wave takes which chunk: with DYN, waves draw chunk numbers from a counter in LDS, so
// a wave that the memory system serves slowly takes fewer chunks and all waves of the
// workgroup finish together (measured: with a fixed interleave the slowest wave of a
// workgroup finishes several microseconds after the average one).  Without DYN wave w
// takes chunks w, w + NW, ...  The order of summation, and so the last bits of the output,
// then depend on timing; the eviction decisions do not involve the attention output.
//
// Loads run D-1 chunks ahead of the arithmetic through a ring of D register stages (the loop
// is unrolled D times, so a stage is a fixed set of registers and nothing is copied).  Loads
// are unconditional: a row past the range re-reads the range's first row and is masked in
// the arithmetic, so the hardware's in-order load counter is all the bookkeeping needed.
//
// Online softmax with slack: a stream keeps its reference value m while no new logit exceeds
// it by more than kSoftmaxSlack (log2 units), so the common chunk needs no rescaling of the
// accumulators; only when some lane of the wave crosses the slack does the wave take the
// rescaling path.  Weights are then at most 2^slack, far inside fp32 range, and the result
// is the same softmax (any reference value gives the same normalised output).
constexpr float kSoftmaxSlack = 16.0f;

// Streaming before the victim is known (single-wave select, below): the slot number travels
// through one LDS word that holds kVictimUnknown until the select wave stores it; a wave logs
// up to kLogCap chunk numbers it consumed in the meantime.
constexpr int kVictimUnknown = 0x7FFFFFFF;
constexpr int kLogCap = 16;
// what the stream does with the one special row of a step (AttnCore::consume)
enum { kRowPlain = 0, kRowSubstitute = 1, kRowExclude = 2 };

template <int HD, int G, bool BF16, int NW, int D, bool DYN>
struct AttnCore {
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int LPR = HD / 8;
  static constexpr int RPW = 64 / LPR;
  static constexpr int NS = NW * RPW;          // softmax streams per workgroup
  static constexpr int U = 2;                  // rows per lane per chunk
  static constexpr int CH = U * RPW;           // rows per chunk
  static constexpr int ROWB = HD * ES;         // bytes per row
  static constexpr int FIRST_DRAW = NW * (D - 1);   // chunks handed out by prime()
  static_assert(D >= 2 && D <= 4, "ring of 2 to 4 stages");

  Raw8<BF16> q[G];
  float m[G], l[G], o[G][8];
  Raw8<BF16> kb[D][U], vb[D][U];
  const char *Kb, *Vb;        // the unit's K and V (wave-uniform)
  uint32_t off0, off_lo;      // byte offsets of the lane's slice in row r0 + rg / in row r0
  int r0;                     // first row of the range (uniform)
  int wave, lane, rg, c;
  float qscale;

  // uq: index of the core's G query heads in units of G heads (= u unless the unit's heads are
  // shared out between workgroups)
  __device__ __forceinline__ void init(const DecodeArgs &a, int u, int tid, int first_row, int uq) {
    lane = tid & 63;
    wave = tid >> 6; c = lane % LPR; rg = lane / LPR;
    qscale = a.qscale;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      q[g].load((const char *)a.q + (((size_t)uq * G + g) * HD + c * 8) * ES);
      m[g] = kNegBig; l[g] = 0.0f;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[g][i] = 0.0f;
    }
    Kb = (const char *)a.K + (size_t)u * a.C * ROWB;
    Vb = (const char *)a.V + (size_t)u * a.C * ROWB;
    r0 = first_row;
    off0 = (uint32_t)(r0 + rg) * ROWB + c * 8 * ES;
    off_lo = (uint32_t)r0 * ROWB + c * 8 * ES;
  }

  // row j of chunk ch, as seen by this lane
  __device__ __forceinline__ int row_of(int ch, int j) const { return r0 + ch * CH + j * RPW + rg; }

  // request chunk `ch` into stage S; rows >= limit are redirected to row r0
  template <int S>
  __device__ __forceinline__ void request(int ch, int limit) {
    uint32_t off[U];
#pragma unroll
    for (int j = 0; j < U; ++j) off[j] = off0 + (uint32_t)ch * (CH * ROWB) + j * (RPW * ROWB);
    if (r0 + (ch + 1) * CH > limit) {   // uniform; only the last chunks of a range
#pragma unroll
      for (int j = 0; j < U; ++j) off[j] = row_of(ch, j) < limit ? off[j] : off_lo;
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      kb[S][j].load(Kb + off[j]);
      vb[S][j].load(Vb + off[j]);
    }
  }

  // request into a stage given by an unrolled loop variable
  __device__ __forceinline__ void request_stage(int s, int ch, int limit) {
    if (s == 0) request<0>(ch, limit);
    if constexpr (D > 1) { if (s == 1) request<1>(ch, limit); }
    if constexpr (D > 2) { if (s == 2) request<2>(ch, limit); }
    if constexpr (D > 3) { if (s == 3) request<3>(ch, limit); }
  }

  // the wave's first D-1 chunks: w, w + NW, ...
  __device__ __forceinline__ void prime(int limit) {
#pragma unroll
    for (int s = 0; s < D - 1; ++s) request_stage(s, wave + s * NW, limit);
  }

  // consume chunk `ch` from stage S.  MASKED: rows >= r1 do not count.  Chunk sub_ch holds row
  // sub_row, which is special: MODE kRowSubstitute takes its K/V from (ksub, vsub) instead of
  // memory, MODE kRowExclude (MASKED form only) leaves it out of the sums.
  template <int S, bool MASKED, int MODE>
  __device__ __forceinline__ void consume(int ch, int r1, int sub_ch, int sub_row,
                                          const Raw8<BF16> &ksub, const Raw8<BF16> &vsub) {
    if constexpr (MODE == kRowSubstitute) {
      if (ch == sub_ch) {   // uniform: one chunk per step
#pragma unroll
        for (int j = 0; j < U; ++j)
          if (row_of(ch, j) == sub_row) { kb[S][j] = ksub; vb[S][j] = vsub; }
      }
    }
#ifdef LSHE_STAGE_LDS
    // Measurement build only (-DLSHE_STAGE_LDS): the chunk goes from the load's registers through
    // LDS and back before it is used, as it would if tiles were staged there -- in the cheapest
    // possible form: every lane writes and reads its own 16-byte pieces (no bank conflicts, no
    // barrier, no second reader).  Compiled out of the shipped library.
    if constexpr (BF16) {
      __shared__ uint4 s_stage[NW * 2 * U * 64];
      uint4 *mine = s_stage + (size_t)wave * (2 * U * 64) + lane;
#pragma unroll
      for (int j = 0; j < U; ++j) { mine[(2 * j) * 64] = kb[S][j].v; mine[(2 * j + 1) * 64] = vb[S][j].v; }
      asm volatile("" ::: "memory");
#pragma unroll
      for (int j = 0; j < U; ++j) { kb[S][j].v = mine[(2 * j) * 64]; vb[S][j].v = mine[(2 * j + 1) * 64]; }
    }
#endif
    bool ok[U];
#pragma unroll
    for (int j = 0; j < U; ++j) ok[j] = !MASKED || row_of(ch, j) < r1;
    if constexpr (MASKED && MODE == kRowExclude) {
#pragma unroll
      for (int j = 0; j < U; ++j) ok[j] = ok[j] && row_of(ch, j) != sub_row;
    }

    float sr[U][G], t[U][G];
    float hi = kNegBig;
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        sr[j][g] = group_sum<LPR>(dot8(q[g], kb[S][j]));
        const float x = fmaf(sr[j][g], qscale, -m[g]);
        t[j][g] = ok[j] ? x : kNegBig;
        hi = fmaxf(hi, t[j][g]);
      }
    if (__builtin_amdgcn_ballot_w64(hi > kSoftmaxSlack) != 0) {   // some stream's reference is stale
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mn = m[g];
#pragma unroll
        for (int j = 0; j < U; ++j) mn = ok[j] ? fmaxf(mn, sr[j][g] * qscale) : mn;
        const float corr = __builtin_amdgcn_exp2f(m[g] - mn);
        m[g] = mn;
        l[g] *= corr;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] *= corr;
#pragma unroll
        for (int j = 0; j < U; ++j) t[j][g] = ok[j] ? fmaf(sr[j][g], qscale, -mn) : kNegBig;
      }
    }
    float p[U][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float ps = 0.0f;
#pragma unroll
      for (int j = 0; j < U; ++j) {
        p[j][g] = __builtin_amdgcn_exp2f(t[j][g]);
        ps = j == 0 ? p[j][g] : ps + p[j][g];
      }
      l[g] += ps;
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      float vf[8];
      vb[S][j].unpack(vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] = fmaf(p[j][g], vf[i], o[g][i]);
    }
  }

  template <bool MASKED, int MODE>
  __device__ __forceinline__ void consume_stage(int s, int ch, int r1, int sub_ch, int sub_row,
                                                const Raw8<BF16> &ksub, const Raw8<BF16> &vsub) {
    if (s == 0) consume<0, MASKED, MODE>(ch, r1, sub_ch, sub_row, ksub, vsub);
    if constexpr (D > 1) { if (s == 1) consume<1, MASKED, MODE>(ch, r1, sub_ch, sub_row, ksub, vsub); }
    if constexpr (D > 2) { if (s == 2) consume<2, MASKED, MODE>(ch, r1, sub_ch, sub_row, ksub, vsub); }
    if constexpr (D > 3) { if (s == 3) consume<3, MASKED, MODE>(ch, r1, sub_ch, sub_row, ksub, vsub); }
  }

  // The wave's next chunk number.  DYN: one lane draws from the LDS counter (which the
  // workgroup set to FIRST_DRAW before its last barrier); the draw is issued a chunk before
  // its value is needed.
  __device__ __forceinline__ uint32_t draw(uint32_t *counter) const {
    uint32_t v = 0;
    if (lane == 0) v = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return v;
  }

  // Stream rows [r0, r1) (prime() already called; r1 > r0).
  template <int MODE>
  __device__ __forceinline__ void stream(int r1, int sub_row, const Raw8<BF16> &ksub,
                                         const Raw8<BF16> &vsub, uint32_t *counter) {
    const int n = r1 - r0;
    const int n_ch = (n + CH - 1) / CH;   // chunks in the range
    const int n_full = n / CH;            // of which whole
    const int sub_ch = sub_row >= r0 ? (sub_row - r0) / CH : -1;
    int id[D];
#pragma unroll
    for (int s = 0; s < D - 1; ++s) id[s] = wave + s * NW;
    id[D - 1] = 0;
    int next_static = wave + (D - 1) * NW;
    uint32_t pending = 0;
    if constexpr (DYN) pending = draw(counter);
    for (;;) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        int nxt;
        if constexpr (DYN) {
          nxt = (int)__builtin_amdgcn_readfirstlane(pending);
          pending = draw(counter);
        } else {
          nxt = next_static;
          next_static += NW;
        }
        id[(s + D - 1) % D] = nxt;
        request_stage((s + D - 1) % D, nxt, r1);
        const int cur = id[s];
        if (cur >= n_ch) return;   // chunk numbers only grow: nothing later is in range either
        // (a chunk with a row to leave out takes the form with per-row conditions)
        if (cur < n_full && !(MODE == kRowExclude && cur == sub_ch))
          consume_stage<false, MODE>(s, cur, r1, sub_ch, sub_row, ksub, vsub);
        else
          consume_stage<true, MODE>(s, cur, r1, sub_ch, sub_row, ksub, vsub);
      }
    }
  }

  // ---- streaming that starts before the victim is known ------------------------------------
  // The waves that do not take part in the select start on the K/V stream at once.  Until the
  // victim's slot appears in *s_e a wave notes the chunks it consumes in `log` (LDS, its own
  // kLogCap entries).  When the slot arrives and its chunk is in the log, the wave consumed the
  // victim's old row: it drops its softmax state and streams the logged chunks again, now with
  // the new token's row in the victim's place (exact: nothing is subtracted).  The other
  // chunks take the substitution in passing.  With the chunk hand-out being dynamic the rest
  // of the workgroup absorbs the few re-read chunks.

  __device__ __forceinline__ static int peek_victim(const int *s_e) {
    return __builtin_amdgcn_readfirstlane(
        __hip_atomic_load(s_e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
  }
  // The select wave stores the slot on every path and waits for nobody, so this ends; the poll
  // count is bounded all the same, so that a mistake elsewhere shows as a status bit and a wrong
  // output, not as waves that never finish: on expiry the caller goes on as if nothing were
  // evicted (kVictimUnknown is returned) after setting LSHE_STATUS_SELECT_TIMEOUT.
  __device__ __forceinline__ int await_victim(const int *s_e, int spin_limit, int32_t *status) const {
    int ev = peek_victim(s_e);
    for (int n = 0; ev == kVictimUnknown && n < spin_limit; ++n) {
      __builtin_amdgcn_s_sleep(8);
      ev = peek_victim(s_e);
    }
    if (ev == kVictimUnknown && lane == 0)
      __hip_atomic_fetch_or(status, LSHE_STATUS_SELECT_TIMEOUT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return ev;
  }

  // After the victim became known: redo the logged chunks if one of them held it.  Stage S
  // must be free (its chunk consumed or out of range).
  template <int S>
  __device__ __forceinline__ void replay(int n_log, const int *log, int r1, int sub_ch, int sub_row,
                                         const Raw8<BF16> &ksub, const Raw8<BF16> &vsub) {
    if (sub_ch < 0) return;
    bool hit = false;
    for (int k = 0; k < n_log; ++k) hit |= log[k] == sub_ch;
    if (!hit) return;   // uniform: the log is the wave's
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = kNegBig; l[g] = 0.0f;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[g][i] = 0.0f;
    }
    for (int k = 0; k < n_log; ++k) {
      const int ch = __builtin_amdgcn_readfirstlane(log[k]);
      request<S>(ch, r1);
      consume<S, true, kRowSubstitute>(ch, r1, sub_ch, sub_row, ksub, vsub);
    }
  }

  // Stream rows [0, r1) (prime() already called; r1 > 0); e_now is the victim's slot if the
  // caller already knows it, else kVictimUnknown.
  __device__ __forceinline__ void stream_deferred(int r1, int e_now, const Raw8<BF16> &ksub,
                                                  const Raw8<BF16> &vsub, uint32_t *counter,
                                                  const int *s_e, int *log, int spin_limit,
                                                  int32_t *status) {
    static_assert(DYN, "deferred streaming draws its chunks");
    const int n = r1 - r0;
    const int n_ch = (n + CH - 1) / CH;
    const int n_full = n / CH;
    bool known = e_now != kVictimUnknown;
    int sub_row = known ? e_now : -1;
    int sub_ch = sub_row >= r0 ? (sub_row - r0) / CH : -1;
    int n_log = 0;
    int id[D];
#pragma unroll
    for (int s = 0; s < D - 1; ++s) id[s] = wave + s * NW;
    id[D - 1] = 0;
    uint32_t pending = draw(counter);
    bool more = true;
    while (more) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        if (s == 0 && !known) {   // once per D chunks: has the victim arrived?  (stage D-1 is free)
          const bool must = n_log + D > kLogCap;   // no room to log another round of chunks
          const int ev = must ? await_victim(s_e, spin_limit, status) : peek_victim(s_e);
          if (ev != kVictimUnknown) {
            known = true;
            sub_row = ev;
            sub_ch = sub_row >= r0 ? (sub_row - r0) / CH : -1;
            replay<D - 1>(n_log, log, r1, sub_ch, sub_row, ksub, vsub);
          } else if (must) {   // the wait expired (status bit set): go on without a victim
            known = true;
          }
        }
        const int nxt = (int)__builtin_amdgcn_readfirstlane(pending);
        pending = draw(counter);
        id[(s + D - 1) % D] = nxt;
        request_stage((s + D - 1) % D, nxt, r1);
        const int cur = id[s];
        if (cur >= n_ch) { more = false; break; }
        if (!known) {
          if (lane == 0) log[n_log] = cur;
          ++n_log;
        }
        if (cur < n_full) consume_stage<false, kRowSubstitute>(s, cur, r1, sub_ch, sub_row, ksub, vsub);
        else consume_stage<true, kRowSubstitute>(s, cur, r1, sub_ch, sub_row, ksub, vsub);
      }
    }
    if (!known) {   // ran out of chunks first: every stage now holds an out-of-range chunk
      sub_row = await_victim(s_e, spin_limit, status);
      if (sub_row != kVictimUnknown) {   // (else the wait expired: status bit set, nothing replayed)
        sub_ch = sub_row >= r0 ? (sub_row - r0) / CH : -1;
        replay<0>(n_log, log, r1, sub_ch, sub_row, ksub, vsub);
      }
    }
  }

  // Fold the softmax state held `XOR` lanes away into this lane's (valid in the lanes whose
  // bit XOR of the lane id is clear).  The partner holds the same head-dim slice of another
  // row group.
  template <int XOR>
  __device__ __forceinline__ void fold_partner() {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m2 = lane_xor<XOR>(m[g]), l2 = lane_xor<XOR>(l[g]);
      const float M = fmaxf(m[g], m2);
      const float w1 = __builtin_amdgcn_exp2f(m[g] - M), w2 = __builtin_amdgcn_exp2f(m2 - M);
      m[g] = M;
      l[g] = l[g] * w1 + l2 * w2;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[g][i] = o[g][i] * w1 + lane_xor<XOR>(o[g][i]) * w2;
    }
  }

  // The wave's four row groups (LPR = 16) summed and written to LDS as the wave's state.  The
  // row groups first agree on one reference per head (two swaps, both results used: every lane
  // gets the maximum) and scale their sums to it; the 9 x G values of a lane (8 output elements
  // and the sum per head) are then added over the row groups two at a time: a swap of the
  // upper half of value A with the lower half of value B followed by one add leaves A's total
  // in the lower lanes and B's in the upper ones, and the same with odd and even rows of 16
  // lanes leaves the totals of four values A, B, C, D in row groups 0, 2, 1, 3.  Three
  // exchanges per four values instead of eight, no copies, and every row group writes a
  // quarter of the state.  With four heads the values are ordered so that row group g ends up
  // with head g whole (two 16-byte writes and the sum); otherwise value 4n + {0, 2, 1, 3}[rg].
  static constexpr int fold_source(int j) {   // which of the 9 x G values goes in as value j
    constexpr int swap12[4] = {0, 2, 1, 3};
    return G == 4 ? swap12[j % 4] * 9 + j / 4 : j;
  }
  __device__ __forceinline__ void fold_rows_to_lds(float (*sm_m)[G], float (*sm_l)[G], float (*sm_o)[G][HD]) {
    static_assert(RPW == 4, "two exchange stages");
    typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
    constexpr int NV = (G * 9 + 3) / 4 * 4;
    float w[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const unsigned x = __float_as_uint(m[g]);
      const u32x2_t h = __builtin_amdgcn_permlane32_swap(x, x, false, false);
      const unsigned y = __float_as_uint(fmaxf(__uint_as_float(h.x), __uint_as_float(h.y)));
      const u32x2_t r = __builtin_amdgcn_permlane16_swap(y, y, false, false);
      const float M = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
      w[g] = __builtin_amdgcn_exp2f(m[g] - M);
      m[g] = M;
    }
    float v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int f = fold_source(j), g = f / 9, e = f - g * 9;
      if (f < G * 9) v[j] = (e < 8 ? o[g][e] : l[g]) * w[g];
      else v[j] = 0.0f;
    }
    float s2[NV / 2];
#pragma unroll
    for (int k = 0; k < NV / 2; ++k) {
      const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[2 * k]), __float_as_uint(v[2 * k + 1]), false, false);
      s2[k] = __uint_as_float(r.x) + __uint_as_float(r.y);
    }
    float t[NV / 4];
#pragma unroll
    for (int n = 0; n < NV / 4; ++n) {
      const u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(s2[2 * n]), __float_as_uint(s2[2 * n + 1]), false, false);
      t[n] = __uint_as_float(r.x) + __uint_as_float(r.y);
    }
    if constexpr (G == 4) {   // row group rg holds head rg
      *(float4 *)&sm_o[wave][rg][c * 8] = make_float4(t[0], t[1], t[2], t[3]);
      *(float4 *)&sm_o[wave][rg][c * 8 + 4] = make_float4(t[4], t[5], t[6], t[7]);
      if (c == 0) sm_l[wave][rg] = t[8];   // (the sum is the same in the 16 lanes of a row)
    } else {
      const int mine = rg == 1 ? 2 : rg == 2 ? 1 : rg;
#pragma unroll
      for (int n = 0; n < NV / 4; ++n) {
        const int j = 4 * n + mine;
        if (j < G * 9) {
          const int g = j / 9, e = j - g * 9;
          if (e < 8) sm_o[wave][g][c * 8 + e] = t[n];
          else if (c == 0) sm_l[wave][g] = t[n];
        }
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) sm_m[wave][g] = m[g];
    }
  }

  // Merge the NS streams.  First the RPW row groups of each wave fold into one state in LDS
  // (cross-lane swaps), then the NW wave states meet in a single round:
  // thread (g, i) sums the NW weighted values of output element i of query head g.
  // final_out: write normalised outputs to a.out; otherwise write the partial state
  // (max, sum, unnormalised output) to `part`.
  // (u: index of the core's heads in units of G heads, as init's uq)
  // part_incl (with part): a second partial state, the first one with one more row folded in
  // whose scaled logits per head are lb_logit[g] and whose value row is lb_v[HD] (lb_logit
  // NULL: no such row, the two states are equal).
  __device__ __forceinline__ void finish(const DecodeArgs &a, int u, int tid, bool final_out,
                                         float *part, const float *vl, float (*sm_m)[G],
                                         float (*sm_l)[G], float (*sm_o)[G][HD],
                                         float *part_incl = nullptr, const float *lb_logit = nullptr,
                                         const float *lb_v = nullptr) {
    if constexpr (RPW == 4) {
      fold_rows_to_lds(sm_m, sm_l, sm_o);
    } else {
      fold_partner<32>();
      fold_partner<16>();
      if constexpr (LPR == 8) fold_partner<8>();
      if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          if (c == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
          *(float4 *)&sm_o[wave][g][c * 8] = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
          *(float4 *)&sm_o[wave][g][c * 8 + 4] = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
        }
      }
    }
    lds_barrier();
    for (int idx = tid; idx < G * HD; idx += 64 * NW) {
      const int g = idx / HD, i = idx - g * HD;
      float M = kNegBig;
#pragma unroll
      for (int k = 0; k < NW; ++k) M = fmaxf(M, sm_m[k][g]);
      float O = 0.0f, Lsum = 0.0f;
#pragma unroll
      for (int k = 0; k < NW; ++k) {
        const float w = __builtin_amdgcn_exp2f(sm_m[k][g] - M);
        O = fmaf(w, sm_o[k][g][i], O);
        Lsum = fmaf(w, sm_l[k][g], Lsum);
      }
      if (final_out) {
        store_out<BF16>(a.out, ((size_t)u * G + g) * HD + i, Lsum > 0.0f ? O / Lsum : 0.0f);
        if (i == 0 && vl) {   // probability on the victim among the new cache plus the victim
          const float pe = __builtin_amdgcn_exp2f(vl[g] - M);
          a.evicted_mass[(size_t)u * G + g] = pe / (Lsum + pe);
        }
      } else {
        part[g * (HD + 2) + 2 + i] = O;
        if (i == 0) { part[g * (HD + 2)] = M; part[g * (HD + 2) + 1] = Lsum; }
        if (part_incl) {
          float M2 = M, L2 = Lsum, O2 = O;
          if (lb_logit) {
            const float x = lb_logit[g];
            M2 = fmaxf(M, x);
            const float we = __builtin_amdgcn_exp2f(M - M2), wx = __builtin_amdgcn_exp2f(x - M2);
            L2 = Lsum * we + wx;
            O2 = O * we + wx * lb_v[i];
          }
          part_incl[g * (HD + 2) + 2 + i] = O2;
          if (i == 0) { part_incl[g * (HD + 2)] = M2; part_incl[g * (HD + 2) + 1] = L2; }
        }
      }
    }
  }
};

// split plan: `S` workgroups per unit over disjoint slot ranges (short ranges: two stages)
constexpr int kAttnStages = 2;
// G is the number of query heads one workgroup carries: the unit's a.G heads go to a.G / G
// workgroups (groups of 8 heads: two workgroups with 4 each), which read the same rows; they
// sit 8 apart in the grid, i.e. on the same XCD and next to each other in dispatch order, so
// that the second reader finds the rows in that XCD's L2.
template <int HD, int G, bool BF16>
__global__ __launch_bounds__(kAttnThreads) void attn_kernel(const DecodeArgs a) {
  constexpr int NW = kAttnThreads / 64;
  typedef AttnCore<HD, G, BF16, NW, kAttnStages, false> Core;
  const int S = a.S, QS = a.G / G;
  int pair = blockIdx.x, qg = 0;   // pair = (unit, split)
  if (QS > 1) {
    const int n_pairs = gridDim.x / QS;
    if (n_pairs % 8 == 0) {
      qg = (blockIdx.x >> 3) % QS;
      pair = (blockIdx.x / (8 * QS)) * 8 + (blockIdx.x & 7);
    } else {
      qg = blockIdx.x % QS;
      pair = blockIdx.x / QS;
    }
  }
  const int u = pair / S, split = pair - u * S;
  const int uq = u * QS + qg;
  const int tid = threadIdx.x;
  const int nv = a.n_valid[u];
  int rps = (nv + S - 1) / S;
  rps = (rps + Core::CH - 1) / Core::CH * Core::CH;
  const int r0 = split * rps;
  const int r1 = min(nv, r0 + rps);

  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ __align__(16) float sm_o[NW][G][HD];
  Core core;
  core.init(a, u, tid, r0, uq);
  if (r1 > r0) {
    const Raw8<BF16> none = {};
    core.prime(r1);
    core.template stream<kRowPlain>(r1, -1, none, none, nullptr);
  }
  core.finish(a, uq, tid, S == 1,
              a.partials + (((size_t)u * S + split) * a.G + qg * G) * (HD + 2),
              a.evicted_mass ? a.victim_logit + (size_t)uq * G : nullptr, sm_m, sm_l, sm_o);
}

// Split plan (few units, so several workgroups per unit over disjoint slot ranges), whole step
// in two launches.  A unit's select needs the whole code table, its attention needs the victim:
// done naively that is three dependent launches (select, attention, merge).  Here every
// attention workgroup selects LOCALLY -- it scores only the code words of its own range and
// finds the range's best candidate (largest summed Hamming distance, lowest slot), which costs
// one short memory round trip and depends on no other workgroup -- and then streams its range
// of the cache as it stands, with that one candidate row set aside.  It writes two partial
// softmax states, without and with the candidate row, the row's logits, and the candidate's
// key.  The merge kernel takes the largest key over the unit's ranges (the global argmax, ties
// to the lowest slot, is the maximum of the local ones), uses the state WITHOUT the row for the
// range that held the victim and the states WITH it for the others, adds the new token's own
// term, and applies Algorithm 1's overwrite (key, value, code, position, count) -- after every
// attention workgroup has finished with the old cache.  Exact: nothing is subtracted.
// G is the number of query heads one workgroup carries (see attn_kernel).
//
// Workspace per (unit, range): [state without the row: a.G x (HD+2)] [state with it: a.G x
// (HD+2)] [the row's scaled logits: a.G] [key: 2 words]; per unit 4 words {occupied slots before
// the step, token index, the new key's code words}.

constexpr int kLocalBatch = 4;   // slots per thread requested together
constexpr int kCombineThreads = 1024;   // workgroup of the merge kernels: one per (unit, query head)
constexpr int kMergePre = 8;   // ranges per thread whose states merge_local_kernel requests before it knows the victim

template <int W, int NT>
struct LocalCodes {
  uint32_t c[kLocalBatch][W];
  int p[kLocalBatch];
  // slots s0, s0 + NT, ... of the range [r0, r1); slots past the end re-read r0 (r1 > r0)
  __device__ __forceinline__ void load(const DecodeArgs &a, int u, int s0, int r0, int r1) {
    const uint32_t *codes = a.code + (size_t)u * a.C * W;
    const int32_t *spos = a.slot_pos + (size_t)u * a.C;
    const bool masked = (a.n_sink | a.n_recent) != 0;
#pragma unroll
    for (int b = 0; b < kLocalBatch; ++b) {
      int s = s0 + b * NT;
      s = s < r1 ? s : r0;
#pragma unroll
      for (int w = 0; w < W; ++w) c[b][w] = codes[(size_t)s * W + w];
      p[b] = masked ? spos[s] : 0;
    }
  }
};

// local_select's scan in the common case -- HashEvict scores, no debug output -- with the group
// size known at compile time: the thread's best key (0: none).  PROTECT: some tokens are kept.
template <int W, int NT, int GT, bool PROTECT>
__device__ __forceinline__ uint32_t local_scan_plain(const DecodeArgs &a, int u, int r0, int r1, int t, int tid,
                                                     LocalCodes<W, NT> &lc, const uint32_t *s_code) {
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t qc[GT][W];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int w = 0; w < W; ++w) qc[g][w] = s_code[g * W + w];
  uint32_t hi = 0;
  for (int s0 = r0 + tid; s0 < r1; s0 += kLocalBatch * NT) {
    if (s0 != r0 + tid) lc.load(a, u, s0, r0, r1);   // (the first batch was requested by the caller)
#pragma unroll
    for (int b = 0; b < kLocalBatch; ++b) {
      const int sl = s0 + b * NT;
      uint32_t sc = 0;
#pragma unroll
      for (int w = 0; w < W; ++w)
#pragma unroll
        for (int g = 0; g < GT; ++g) sc += __popc(lc.c[b][w] ^ qc[g][w]);
      bool ok = sl < r1;
      if constexpr (PROTECT) ok = ok && lc.p[b] >= a.n_sink && lc.p[b] <= newest_evictable;
      const uint32_t key = ok ? make_key(sc, (uint32_t)sl) : 0u;
      hi = hi > key ? hi : key;
    }
  }
  return hi;
}

// The best candidate among the slots [r0, r1) of unit u, as a key of two words that orders like
// the selection rule: HashEvict (score + 1) << 20 | (0xFFFFF - slot) and 0; L2-norm policy norm
// bits + 1 and 0xFFFFF - slot; (0, 0) if no slot of the range may be evicted.  Every thread gets
// the key.  s_best: 2 * NT/64 words.
template <int W, int NT>
__device__ __forceinline__ void local_select(const DecodeArgs &a, int u, int r0, int r1, int t, int tid,
                                             LocalCodes<W, NT> &lc, const uint32_t *s_code,
                                             uint32_t *s_best, uint32_t &k0, uint32_t &k1) {
  constexpr int NWAVES = NT / 64;
  const int C = a.C, G = a.G, lane = tid & 63, wave = tid >> 6;
  const bool l2 = W == 1 && a.policy == LSHE_POLICY_L2NORM;
  const bool masked = (a.n_sink | a.n_recent) != 0;
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t hi = 0, lo = 0;
  const bool plain = !l2 && a.scores_dbg == nullptr;
  if (plain) {
#define LSHE_LOCAL_SCAN(GT_)                                                                              \
  hi = masked ? local_scan_plain<W, NT, GT_, true>(a, u, r0, r1, t, tid, lc, s_code)                      \
              : local_scan_plain<W, NT, GT_, false>(a, u, r0, r1, t, tid, lc, s_code)
    switch (G) {
      case 1: LSHE_LOCAL_SCAN(1); break;
      case 2: LSHE_LOCAL_SCAN(2); break;
      case 4: LSHE_LOCAL_SCAN(4); break;
      default: LSHE_LOCAL_SCAN(8); break;
    }
#undef LSHE_LOCAL_SCAN
  }
  for (int s0 = r0 + tid; !plain && s0 < r1; s0 += kLocalBatch * NT) {
    if (s0 != r0 + tid) lc.load(a, u, s0, r0, r1);   // (the first batch was requested by the caller)
#pragma unroll
    for (int b = 0; b < kLocalBatch; ++b) {
      const int sl = s0 + b * NT;
      if (sl < r1) {
        const bool ok = !masked || (lc.p[b] >= a.n_sink && lc.p[b] <= newest_evictable);
        if (l2) {
          const uint32_t v = lc.c[b][0];
          if (a.scores_dbg) a.scores_dbg[(size_t)u * C + sl] = (int32_t)v;
          const uint32_t h = ok ? v + 1u : 0u;
          if (h > hi) { hi = h; lo = 0xFFFFFu - (uint32_t)sl; }   // ascending slots per thread
        } else {
          uint32_t sc = 0;
#pragma unroll
          for (int w = 0; w < W; ++w)
            for (int g = 0; g < G; ++g) sc += __popc(lc.c[b][w] ^ s_code[g * W + w]);
          if (a.scores_dbg) a.scores_dbg[(size_t)u * C + sl] = (int32_t)sc;
          const uint32_t key = ok ? make_key(sc, (uint32_t)sl) : 0u;
          hi = hi > key ? hi : key;
        }
      }
    }
  }
  const uint32_t whi = wave_max_u32(hi);
  const uint32_t wlo = l2 ? wave_max_u32(hi == whi ? lo : 0u) : 0u;
  if (lane == 0) { s_best[wave] = whi; s_best[NWAVES + wave] = wlo; }
  lds_barrier();
  k0 = 0; k1 = 0;
#pragma unroll
  for (int k = 0; k < NWAVES; ++k) {
    const uint32_t h = s_best[k], l = s_best[NWAVES + k];
    if (h > k0 || (h == k0 && l > k1)) { k0 = h; k1 = l; }
  }
}

// Register stages of this kernel's K/V stream and how chunks are shared out.  Four stages and a
// run-time draw from an LDS counter were both measured on the long-context step and are slower
// than two stages over a fixed interleave: the first chunk is requested before the select phase
// waits for anything, so the memory system is not idle during it, and with ranges of a few
// hundred slots the draw's extra LDS round trip per chunk costs more than the imbalance it evens.
constexpr int kLocalStages = 2;
constexpr bool kLocalDraw = false;

template <int HD, int G, int W, bool BF16>
__global__ __launch_bounds__(kAttnThreads) void attn_local_kernel(const DecodeArgs a0) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int NT = kAttnThreads, NW = NT / 64, LPR = HD / 8;
  typedef AttnCore<HD, G, BF16, NW, kLocalStages, kLocalDraw> Core;
  const int S = a0.S, QS = a0.G / G;
  int pair = blockIdx.x, qg = 0;
  if (QS > 1) {
    const int n_pairs = gridDim.x / QS;
    if (n_pairs % 8 == 0) {
      qg = (blockIdx.x >> 3) % QS;
      pair = (blockIdx.x / (8 * QS)) * 8 + (blockIdx.x & 7);
    } else {
      qg = blockIdx.x % QS;
      pair = blockIdx.x / QS;
    }
  }
  const int u = pair / S, split = pair - u * S;
  const int uq = u * QS + qg;
  const int tid = threadIdx.x;
  DecodeArgs a = a0;
  if (split != 0 || qg != 0) a.codes_dbg = nullptr;   // one copy of the debug outputs
  if (qg != 0) a.scores_dbg = nullptr;

  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];
  __shared__ uint32_t s_best[2 * NW];
  __shared__ uint32_t s_next;                   // next chunk of the K/V stream to hand out
  __shared__ float s_lbl[G];                    // the set-aside row's scaled logits (this workgroup's heads)
  __shared__ __align__(16) float s_lbv[HD];     // ... and its value row
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ __align__(16) float sm_o[NW][G][HD];

  LSHE_STAMP(0);
  // The slot ranges are cut from the budget, not from the occupied count, so that nothing at the
  // workgroup's start waits for n_valid: every row below the budget is a valid address, and what
  // turns out to be unoccupied is masked when it is used (a cache that is still filling leaves the
  // last ranges short or empty; a full one, the usual state when decoding, loses nothing).
  int rps = (a.C + S - 1) / S;
  rps = (rps + Core::CH - 1) / Core::CH * Core::CH;
  const int r0 = split * rps;
  const int r1c = min(a.C, r0 + rps);
  const bool anyc = r1c > r0;   // (rounding the range length up can leave the last ranges empty)
  // every request of the workgroup's start goes out before anything waits: the range's code
  // words, the step inputs and R (wave 0), the query pieces, the first chunks of the stream
  LocalCodes<W, NT> lc;
  if (anyc) lc.load(a, u, r0 + tid, r0, r1c);
  StepHash<HD, W, BF16> hash;
  if (tid < 64) hash.issue(a, u, tid);
  Core core;
  core.init(a, u, tid, r0, uq);
  if (anyc) core.prime(r1c);
  const int nv = a.n_valid[u];                  // occupied slots before the step
  const int t = a.pos[u / a.units_per_seq];
  LSHE_STAMP(1);
  if (tid < 64) hash.finish(a, u, tid, s_code);
  if (tid == 64) s_next = Core::FIRST_DRAW;
  const int r1 = min(nv, r1c);
  const bool any = r1 > r0;     // (implies anyc)
  LSHE_STAMP(2);
  lds_barrier();   // the codes of the step inputs are in s_code
  LSHE_STAMP(3);

  uint32_t k0 = 0, k1 = 0;
  if (any) local_select<W, NT>(a, u, r0, r1, t, tid, lc, s_code, s_best, k0, k1);   // (uniform condition)
  LSHE_STAMP(7);
  if (a.scores_dbg && split == 0)
    for (int sl = nv + tid; sl < a.C; sl += NT) a.scores_dbg[(size_t)u * a.C + sl] = -1;
  const bool evicting = nv == a.C;
  if (!evicting) { k0 = 0; k1 = 0; }   // a filling cache evicts nothing
  const bool l2 = W == 1 && a.policy == LSHE_POLICY_L2NORM;
  const int lb = k0 != 0u ? (l2 ? (int)(0xFFFFFu - k1) : key_slot(k0)) : -1;

  // the candidate row's own term, taken from the cache as it stands: requested now, used after
  // the stream (loads return in order, so nothing waits for it)
  Raw8<BF16> lbk = {}, lbv = {};
  if (lb >= 0) {
    if (tid < LPR) lbk.load((const char *)a.K + (((size_t)u * a.C + lb) * HD + tid * 8) * ES);
    else if (tid >= 64 && tid < 64 + LPR)
      lbv.load((const char *)a.V + (((size_t)u * a.C + lb) * HD + (tid - 64) * 8) * ES);
  }
  LSHE_STAMP(4);
  if (any) {
    const Raw8<BF16> none = {};
    core.template stream<kRowExclude>(r1, lb, none, none, &s_next);
  }
  LSHE_STAMP(5);
  if (lb >= 0) {
    if (tid < LPR) {   // lane c of wave 0 holds piece c of every query head
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float x = group_sum<LPR>(dot8(core.q[g], lbk)) * a.qscale;
        if (tid == 0) s_lbl[g] = x;
      }
    } else if (tid >= 64 && tid < 64 + LPR) {
      float vf[8];
      lbv.unpack(vf);
#pragma unroll
      for (int i = 0; i < 8; ++i) s_lbv[(tid - 64) * 8 + i] = vf[i];
    }
  }
  float *part = a.partials + ((size_t)u * S + split) * local_part_floats(a.G, HD);
  // (finish() has a barrier between these LDS writes and its reads of s_lbl / s_lbv)
  core.finish(a, uq, tid, false, part + qg * G * (HD + 2), nullptr, sm_m, sm_l, sm_o,
              part + (a.G + qg * G) * (HD + 2), lb >= 0 ? s_lbl : nullptr, s_lbv);
  LSHE_STAMP(6);
  {
    float *tail = part + 2 * a.G * (HD + 2);
    if (tid < G) tail[qg * G + tid] = lb >= 0 ? s_lbl[tid] : kNegBig;
  }
  if (qg == 0) {
    float *tail = part + 2 * a.G * (HD + 2);
    if (tid == 64) { ((uint32_t *)tail)[a.G] = k0; ((uint32_t *)tail)[a.G + 1] = k1; }
    if (split == 0) {
      int32_t *so = a.sel_out + (size_t)u * 4;
      if (tid == 128) { so[0] = nv; so[1] = t; }
      if (tid >= 129 && tid < 129 + W) so[2 + (tid - 129)] = (int32_t)s_code[a.G * W + (tid - 129)];
    }
  }
}

// Second launch of that plan: one workgroup of 1024 threads per (unit, query head).  (Letting
// every wave work out the victim and the weights on its own, with wave reductions and no
// barriers, was tried: sixteen-fold redundant loads made it three times slower at 256 workgroups.)
template <int HD, bool BF16>
__global__ __launch_bounds__(kCombineThreads) void merge_local_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int NG = kCombineThreads / HD, LPR = HD / 8, NWV = kCombineThreads / 64;
  const int G = a.G, S = a.S, C = a.C, PS = local_part_floats(G, HD), INCL = G * (HD + 2);
  const int u = blockIdx.x / G, g = blockIdx.x - u * G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *pu = a.partials + (size_t)u * S * PS;
  const int32_t *so = a.sel_out + (size_t)u * 4;
  const bool l2 = a.policy == LSHE_POLICY_L2NORM;

  __shared__ float s_red[NWV];
  __shared__ uint32_t s_key[2 * NWV];
  __shared__ float s_M, s_L, s_xnew;
  __shared__ int s_rstar;
  __shared__ float s_o[NG][HD];
  __shared__ float s_w[256];   // weights of the ranges (S <= 256)

  // Everything a thread needs from the partials -- both forms of every state -- is requested
  // before anything waits: the kernel is one memory round trip and a few LDS reductions.
  LSHE_STAMP(8);
  const int nv = so[0], t = so[1];
  // (what the overwrite at the end stores is requested here too: see merge_small_kernel)
  constexpr int VEC = HD * ES / 16;
  uint4 new_piece = {};
  uint32_t new_code = 0;
  if (g == 0) {
    if (tid < VEC) new_piece = ((const uint4 *)((const char *)a.k_new + (size_t)u * HD * ES))[tid];
    else if (tid >= 64 && tid < 64 + VEC)
      new_piece = ((const uint4 *)((const char *)a.v_new + (size_t)u * HD * ES))[tid - 64];
    else if (tid >= 128 && tid < 128 + 2) new_code = (uint32_t)so[2 + (tid - 128)];
  }
  uint32_t k0 = 0, k1 = 0;
  float me = kNegBig, le = 0.0f, mi = kNegBig, li = 0.0f;   // thread k: (max, sum) without / with the row
  if (tid < S) {
    const float *pk = pu + (size_t)tid * PS;
    k0 = ((const uint32_t *)pk)[2 * INCL + G];
    k1 = ((const uint32_t *)pk)[2 * INCL + G + 1];
    me = pk[g * (HD + 2)]; le = pk[g * (HD + 2) + 1];
    mi = pk[INCL + g * (HD + 2)]; li = pk[INCL + g * (HD + 2) + 1];
  }
  // thread (grp, i): element i of the states of ranges grp, grp + NG, ..., both forms
  const int grp = tid / HD, i = tid - grp * HD;
  float oe[kMergePre], oi[kMergePre];
#pragma unroll
  for (int j = 0; j < kMergePre; ++j) {
    const int k = grp + j * NG;
    if (k < S) {   // (uniform per wave)
      const float *pk = pu + (size_t)k * PS + g * (HD + 2) + 2 + i;
      oe[j] = pk[0];
      oi[j] = pk[INCL];
    } else {
      oe[j] = 0.0f; oi[j] = 0.0f;
    }
  }
  // the new token's own logit (eq. 1 scaling): one group of lanes of the last wave
  if (wave == NWV - 1) {
    const int c = lane % LPR;
    Raw8<BF16> q, k;
    q.load((const char *)a.q + (((size_t)u * G + g) * HD + c * 8) * ES);
    k.load((const char *)a.k_new + ((size_t)u * HD + c * 8) * ES);
    const float x = group_sum<LPR>(dot8(q, k)) * a.qscale;
    if (lane == 0) s_xnew = x;
  }
  float vn = 0.0f;   // the new token's value element (threads that write the output)
  if (tid < HD) {
    if constexpr (BF16) vn = __uint_as_float((uint32_t)((const uint16_t *)a.v_new)[(size_t)u * HD + tid] << 16);
    else vn = ((const float *)a.v_new)[(size_t)u * HD + tid];
  }
  if (tid == 0) s_rstar = -1;

  // ---- the victim: the largest local key (S <= 256: one key per thread) ---------------------------
  const uint32_t w0 = wave_max_u32(k0);
  const uint32_t w1 = wave_max_u32(k0 == w0 ? k1 : 0u);
  if (lane == 0) { s_key[wave] = w0; s_key[NWV + wave] = w1; }
  __syncthreads();
  uint32_t K0 = 0, K1 = 0;
#pragma unroll
  for (int k = 0; k < NWV; ++k) {
    const uint32_t h = s_key[k], l = s_key[NWV + k];
    if (h > K0 || (h == K0 && l > K1)) { K0 = h; K1 = l; }
  }
  if (tid < S && K0 != 0u && k0 == K0 && k1 == K1) s_rstar = tid;   // keys hold the slot: one thread
  LSHE_STAMP(9);
  __syncthreads();
  const int rstar = s_rstar;
  const bool evicting = nv == C;
  const int e = evicting ? (rstar >= 0 ? (l2 ? (int)(0xFFFFFu - K1) : key_slot(K0)) : -1) : nv;

  // ---- softmax merge: the state without its candidate row for the victim's range, with it for the
  //      others, plus the new token (a full cache with nothing evictable -- no valid configuration
  //      has one -- takes no new token) ----------------------------------------------------------------
  const float xnew = (evicting && rstar < 0) ? kNegBig : s_xnew;
  const bool mine_excl = tid == rstar;
  const float mk = mine_excl ? me : mi, lk = mine_excl ? le : li;
  float mx = mk;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  float M = xnew;
#pragma unroll
  for (int k = 0; k < NWV; ++k) M = fmaxf(M, s_red[k]);   // (every thread: no second round through LDS)
  const float w = tid < S ? __builtin_amdgcn_exp2f(mk - M) : 0.0f;
  if (tid < S) s_w[tid] = w;
  float ls = w * lk;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ls += __shfl_xor(ls, off);
  __syncthreads();            // every thread has read s_red
  if (lane == 0) s_red[wave] = ls;
  __syncthreads();            // also publishes s_w
  const float wnew = __builtin_amdgcn_exp2f(xnew - M);
  float O = 0.0f;
#pragma unroll
  for (int j = 0; j < kMergePre; ++j) {
    const int k = grp + j * NG;
    if (k < S) O = fmaf(s_w[k], k == rstar ? oe[j] : oi[j], O);
  }
#pragma unroll 4
  for (int k = grp + kMergePre * NG; k < S; k += NG)   // (more ranges than the registers hold)
    O = fmaf(s_w[k], pu[(size_t)k * PS + (k == rstar ? 0 : INCL) + g * (HD + 2) + 2 + i], O);
  s_o[grp][i] = O;
  __syncthreads();
  if (tid < HD) {
    float o = 0.0f, L = wnew;
#pragma unroll
    for (int j = 0; j < NG; ++j) o += s_o[j][tid];
#pragma unroll
    for (int k = 0; k < NWV; ++k) L += s_red[k];
    o = fmaf(wnew, vn, o);
    store_out<BF16>(a.out, ((size_t)u * G + g) * HD + tid, L > 0.0f ? o / L : 0.0f);
    if (tid == 0 && a.evicted_mass) {
      float mass = 0.0f;
      if (evicting && rstar >= 0) {
        const float vl = pu[(size_t)rstar * PS + 2 * INCL + g];
        const float pe = __builtin_amdgcn_exp2f(vl - M);
        mass = pe / (L + pe);
      }
      a.evicted_mass[(size_t)u * G + g] = mass;
    }
  }
  // ---- Algorithm 1 steps 2-5, now that no workgroup reads the old cache any more --------------------
  if (g == 0) {
    const int W = l2 ? 1 : (a.r + 31) / 32;
    if (e >= 0) {
      if (tid < VEC) ((uint4 *)((char *)a.K + ((size_t)u * C + e) * HD * ES))[tid] = new_piece;
      else if (tid >= 64 && tid < 64 + VEC) ((uint4 *)((char *)a.V + ((size_t)u * C + e) * HD * ES))[tid - 64] = new_piece;
      else if (tid >= 128 && tid < 128 + W) a.code[((size_t)u * C + e) * W + (tid - 128)] = new_code;
      else if (tid == 192) {
        a.slot_pos[(size_t)u * C + e] = t;
        if (nv < C) a.n_valid[u] = nv + 1;
      }
    }
    if (tid == 193 && a.evicted) a.evicted[u] = e;
  }
  LSHE_STAMP(10);
}

// The same merge when a unit has at most kMergeSmallRanges slot ranges (per-layer calls, the
// long-context configuration): one workgroup of HD threads per (unit, query head), thread i
// owning output element i, and no barrier at all.  Every wave works out the victim, the
// reference maximum and the weights on its own from the ranges' keys and (max, sum) pairs --
// lane k takes range k; a few dozen redundant 4-byte loads -- and a thread reads element i of
// both forms of every range's state before anything waits, so the kernel is one memory round
// trip, two wave reductions and S multiply-adds.

static_assert(kMergeSmallRanges <= 32, "merge_small_kernel reduces over the first two rows of 16 lanes");
template <int HD, bool BF16>
__global__ __launch_bounds__(HD) void merge_small_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4, LPR = HD / 8, VEC = HD * ES / 16;
  const int G = a.G, S = a.S, C = a.C, PS = local_part_floats(G, HD), INCL = G * (HD + 2);
  const int u = blockIdx.x / G, g = blockIdx.x - u * G;
  const int tid = threadIdx.x, lane = tid & 63;
  const float *pu = a.partials + (size_t)u * S * PS;
  const int32_t *so = a.sel_out + (size_t)u * 4;
  const bool l2 = a.policy == LSHE_POLICY_L2NORM;

  LSHE_STAMP(8);
  const int nv = so[0], t = so[1];
  // what Algorithm 1's overwrite stores, requested with everything else so that the kernel's
  // last act is stores only (threads of head 0: key pieces, value pieces, the key's code words)
  uint4 new_piece = {};
  uint32_t new_code = 0;
  if (g == 0) {
    if (tid < VEC) new_piece = ((const uint4 *)((const char *)a.k_new + (size_t)u * HD * ES))[tid];
    else if (tid < 2 * VEC) new_piece = ((const uint4 *)((const char *)a.v_new + (size_t)u * HD * ES))[tid - VEC];
    else if (tid < 2 * VEC + 2) new_code = (uint32_t)so[2 + (tid - 2 * VEC)];
  }
  uint32_t k0 = 0, k1 = 0;
  float me = kNegBig, le = 0.0f, mi = kNegBig, li = 0.0f;   // lane k: (max, sum) without / with the row
  if (lane < S) {
    const float *pk = pu + (size_t)lane * PS;
    k0 = ((const uint32_t *)pk)[2 * INCL + G];
    k1 = ((const uint32_t *)pk)[2 * INCL + G + 1];
    me = pk[g * (HD + 2)]; le = pk[g * (HD + 2) + 1];
    mi = pk[INCL + g * (HD + 2)]; li = pk[INCL + g * (HD + 2) + 1];
  }
  float oe[kMergeSmallRanges], oi[kMergeSmallRanges];
#pragma unroll
  for (int k = 0; k < kMergeSmallRanges; ++k) {
    if (k < S) {   // (uniform)
      const float *pk = pu + (size_t)k * PS + g * (HD + 2) + 2 + tid;
      oe[k] = pk[0];
      oi[k] = pk[INCL];
    } else {
      oe[k] = 0.0f; oi[k] = 0.0f;
    }
  }
  // the new token's own logit (eq. 1 scaling) and value element
  float xn;
  {
    const int c = lane % LPR;
    Raw8<BF16> q, k;
    q.load((const char *)a.q + (((size_t)u * G + g) * HD + c * 8) * ES);
    k.load((const char *)a.k_new + ((size_t)u * HD + c * 8) * ES);
    xn = group_sum<LPR>(dot8(q, k)) * a.qscale;
  }
  float vn;
  if constexpr (BF16) vn = __uint_as_float((uint32_t)((const uint16_t *)a.v_new)[(size_t)u * HD + tid] << 16);
  else vn = ((const float *)a.v_new)[(size_t)u * HD + tid];

  // ---- the victim: the largest local key -------------------------------------------------------------
  const uint32_t K0 = wave_max_u32(k0);
  const uint32_t K1 = wave_max_u32(k0 == K0 ? k1 : 0u);
  const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < S && K0 != 0u && k0 == K0 && k1 == K1);
  const int rstar = hit != 0 ? (int)__builtin_ctzll(hit) : -1;   // keys hold the slot: one lane
  LSHE_STAMP(9);
  const bool evicting = nv == C;
  const int e = evicting ? (rstar >= 0 ? (l2 ? (int)(0xFFFFFu - K1) : key_slot(K0)) : -1) : nv;

  // ---- softmax merge: the state without its candidate row for the victim's range, with it for the
  //      others, plus the new token (a full cache with nothing evictable takes no new token) ------------
  const float xnew = (evicting && rstar < 0)
                         ? kNegBig
                         : __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(xn)));
  const bool mine_excl = lane == rstar;
  const float mk = mine_excl ? me : mi, lk = mine_excl ? le : li;
  // reductions over the ranges (lanes 0 .. S-1 <= 31: the first two rows of 16 lanes) with
  // register-level lane exchanges; a butterfly of LDS permutes costs a round trip per stage
  auto lane_f32 = [](float x, int l) __attribute__((always_inline)) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), l));
  };
  float M = mk;
  M = fmaxf(M, dpp_f32<kDppQuadSwap1>(M));
  M = fmaxf(M, dpp_f32<kDppQuadSwap2>(M));
  M = fmaxf(M, dpp_f32<kDppRowHalfMirror>(M));
  M = fmaxf(M, dpp_f32<kDppRowMirror>(M));
  M = fmaxf(fmaxf(lane_f32(M, 0), lane_f32(M, 16)), xnew);
  const float w = lane < S ? __builtin_amdgcn_exp2f(mk - M) : 0.0f;
  float L = group_sum<16>(w * lk);
  L = lane_f32(L, 0) + lane_f32(L, 16);
  const float wnew = __builtin_amdgcn_exp2f(xnew - M);
  L += wnew;
  float O = wnew * vn;
#pragma unroll
  for (int k = 0; k < kMergeSmallRanges; ++k) {
    if (k < S) {
      const float wk = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(w), k));
      O = fmaf(wk, k == rstar ? oe[k] : oi[k], O);
    }
  }
  store_out<BF16>(a.out, ((size_t)u * G + g) * HD + tid, L > 0.0f ? O / L : 0.0f);
  if (tid == 0 && a.evicted_mass) {
    float mass = 0.0f;
    if (evicting && rstar >= 0) {
      const float vl = pu[(size_t)rstar * PS + 2 * INCL + g];
      const float pe = __builtin_amdgcn_exp2f(vl - M);
      mass = pe / (L + pe);
    }
    a.evicted_mass[(size_t)u * G + g] = mass;
  }
  // ---- Algorithm 1 steps 2-5, now that no workgroup reads the old cache any more --------------------
  if (g == 0) {
    const int W = l2 ? 1 : (a.r + 31) / 32;
    if (e >= 0) {
      if (tid < VEC) ((uint4 *)((char *)a.K + ((size_t)u * C + e) * HD * ES))[tid] = new_piece;
      else if (tid < 2 * VEC) ((uint4 *)((char *)a.V + ((size_t)u * C + e) * HD * ES))[tid - VEC] = new_piece;
      else if (tid < 2 * VEC + W) a.code[((size_t)u * C + e) * W + (tid - 2 * VEC)] = new_code;
      else if (tid == 2 * VEC + 2) {
        a.slot_pos[(size_t)u * C + e] = t;
        if (nv < C) a.n_valid[u] = nv + 1;
      }
    }
    if (tid == 2 * VEC + 3 && a.evicted) a.evicted[u] = e;
  }
  LSHE_STAMP(10);
}

// Merge the S partial softmax states (split plan, S > 1).  One workgroup of 1024 threads per
// (unit, query head): thread k first turns partial k's (max, sum) into a weight, then
// 1024/HD thread groups each sum every (1024/HD)-th weighted partial output, and LDS adds
// the groups.  All loads of a thread are independent, so S = 150 partials cost a few
// memory round trips, not 150.

template <int HD, bool BF16>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const DecodeArgs a) {
  constexpr int NG = kCombineThreads / HD;   // thread groups
  const int G = a.G, S = a.S;
  const int u = blockIdx.x / G, g = blockIdx.x - u * G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *pu = a.partials + ((size_t)u * S * G + g) * (HD + 2);   // partial k at + k*G*(HD+2)
  const size_t kstride = (size_t)G * (HD + 2);

  __shared__ float s_red[kCombineThreads / 64];
  __shared__ float s_M, s_L;
  __shared__ float s_o[NG][HD];
  extern __shared__ float s_w[];   // [S] weights

  // global max of the partial maxima
  float mx = kNegBig;
  for (int k = tid; k < S; k += kCombineThreads) mx = fmaxf(mx, pu[k * kstride]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    float m = s_red[0];
    for (int i = 1; i < kCombineThreads / 64; ++i) m = fmaxf(m, s_red[i]);
    s_M = m;
  }
  __syncthreads();
  const float M = s_M;
  // weights and the weighted sum of the partial sums
  float ls = 0.0f;
  for (int k = tid; k < S; k += kCombineThreads) {
    const float w = __builtin_amdgcn_exp2f(pu[k * kstride] - M);
    s_w[k] = w;
    ls = fmaf(w, pu[k * kstride + 1], ls);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ls += __shfl_xor(ls, off);
  __syncthreads();            // s_red readers of the first round are done
  if (lane == 0) s_red[wave] = ls;
  __syncthreads();            // also publishes s_w
  if (tid == 0) {
    float l = 0.0f;
    for (int i = 0; i < kCombineThreads / 64; ++i) l += s_red[i];
    s_L = l;
  }
  // weighted sum of the partial outputs
  const int grp = tid / HD, i = tid - grp * HD;
  float O = 0.0f;
#pragma unroll 4
  for (int k = grp; k < S; k += NG) O = fmaf(s_w[k], pu[k * kstride + 2 + i], O);
  s_o[grp][i] = O;
  __syncthreads();
  if (tid < HD) {
    float o = 0.0f;
#pragma unroll
    for (int j = 0; j < NG; ++j) o += s_o[j][tid];
    const float L = s_L;
    store_out<BF16>(a.out, ((size_t)u * G + g) * HD + tid, L > 0.0f ? o / L : 0.0f);
    if (tid == 0 && a.evicted_mass) {
      const float pe = __builtin_amdgcn_exp2f(a.victim_logit[(size_t)u * G + g] - M);
      a.evicted_mass[(size_t)u * G + g] = pe / (L + pe);
    }
  }
}

// fused plan: the whole step of one unit in one workgroup of NW waves
template <int HD, int G, int W, bool BF16, int NW, int D>
__global__ __launch_bounds__(64 * NW) void decode_fused_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int NT = 64 * NW;
  typedef AttnCore<HD, G, BF16, NW, D, true> Core;
  const int u = blockIdx.x, tid = threadIdx.x;

  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];
  __shared__ uint32_t s_best[2 * NW];
  __shared__ uint32_t s_next;   // next chunk of the K/V stream to hand out
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ __align__(16) float sm_o[NW][G][HD];

  // Request order matters: the small loads the select phase waits on (step inputs, R, the
  // code table) go out first, the bulk K/V rows after them, so the select phase is not queued
  // behind the stream it is meant to hide under.
  const int nv = a.n_valid[u];
  const int t = a.pos[u / a.units_per_seq];
  CodePrefetch<W, NT> pre;
  pre.load(a, u, tid);
  if (tid < 64) hash_step_inputs<HD, W, BF16>(a, u, tid, s_code);
  if (tid == 64) s_next = Core::FIRST_DRAW;
  Core core;
  core.init(a, u, tid, 0, u);
  // the lane's slices of the new key and value: they stand in for slot e in the stream
  Raw8<BF16> ksub, vsub;
  ksub.load((const char *)a.k_new + ((size_t)u * HD + core.c * 8) * ES);
  vsub.load((const char *)a.v_new + ((size_t)u * HD + core.c * 8) * ES);
  // First blocks of the stream, requested before the victim (or even n_valid) is known: any
  // row below the budget is a valid address; rows that turn out to be unoccupied are masked
  // when the block is consumed, and whatever is loaded for the victim's row is replaced.
  core.prime(a.C);

  lds_barrier();
  int e;
  if constexpr (W == 1) {
    e = a.policy == LSHE_POLICY_L2NORM ? select_l2<NT>(a, u, nv, t, tid, pre, s_best)
                                       : score_and_select<W, NT>(a, u, nv, t, tid, pre, s_code, s_best);
  } else {
    e = score_and_select<W, NT>(a, u, nv, t, tid, pre, s_code, s_best);
  }
  __shared__ float s_vl[kMaxGroup];
  if (a.evicted_mass) {   // read the victim's key before it is overwritten
    victim_logits<HD, BF16>(a, u, e, nv == a.C && e >= 0, tid, s_vl);
    lds_barrier();
  }
  overwrite_slot<HD, W, BF16>(a, u, e, nv, t, tid, s_code);

  const int r1 = (nv < a.C && e >= 0) ? nv + 1 : nv;
  if (r1 > 0) core.template stream<kRowSubstitute>(r1, e, ksub, vsub, &s_next);
  core.finish(a, u, tid, true, nullptr, a.evicted_mass ? s_vl : nullptr, sm_m, sm_l, sm_o);
}

// ---- fused plan, single-wave select ---------------------------------------------------------
// When the unit's code table is small enough for one wave to score from registers, wave 0
// does the whole select (hash, score, argmax, overwrite) on its own while the other waves
// are already streaming K/V; they pick the victim's slot up from LDS when it appears (see
// stream_deferred).  The select then costs the step one wave's time, not a stall of all.
// Wave 0 only.  issue() requests everything the select reads (the unit's whole code table,
// the positions if some tokens are protected, the step inputs and R) before anything waits;
// finish() returns the slot to write (as score_and_select / select_l2 do) after storing it to
// *s_e, taking the victim's logits if asked, and overwriting the slot.
template <int HD, int G, int W, bool BF16>
struct SoloSelect {
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int MAXV = kSoloMaxWords / 256;
  static constexpr int SPV = 4 / W;   // slots per 16-byte vector of the code table
  uint4 v[MAXV];
  int pp[MAXV][SPV];
  StepHash<HD, W, BF16> hash;

  __device__ __forceinline__ void issue(const DecodeArgs &a, int u, int lane) {
    const int C = a.C;
    const bool masked = (a.n_sink | a.n_recent) != 0;
    const int nvec = C * W / 4;
    const uint4 *cv = (const uint4 *)(a.code + (size_t)u * C * W);
    const int32_t *spos = a.slot_pos + (size_t)u * C;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      const int q = j * 64 + lane;
      v[j] = cv[q < nvec ? q : 0];
    }
    if (masked) {
#pragma unroll
      for (int j = 0; j < MAXV; ++j) {
        const int q = j * 64 + lane;
        const int32_t *pq = spos + (size_t)(q < nvec ? q : 0) * SPV;
        if constexpr (W == 1) {
          const int4 x = *(const int4 *)pq;
          pp[j][0] = x.x; pp[j][1] = x.y; pp[j][2] = x.z; pp[j][3] = x.w;
        } else {
          const int2 x = *(const int2 *)pq;
          pp[j][0] = x.x; pp[j][1] = x.y;
        }
      }
    }
    hash.issue(a, u, lane);
  }

  // The scan of a full cache under HashEvict scores with no debug output, without the per-slot
  // branches of the general form in finish(): the lane's best key (0: none).  PROTECT: some
  // tokens are kept (first n_sink, last n_recent), positions in pp.
  template <bool PROTECT>
  __device__ __forceinline__ uint32_t compact_scan(const DecodeArgs &a, int t, int lane,
                                                   const uint32_t *s_code) const {
    uint32_t qc[G][W];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int w = 0; w < W; ++w) qc[g][w] = s_code[g * W + w];
    const int nvec = a.C * W / 4;
    const int newest_evictable = t - 1 - a.n_recent;
    uint32_t best = 0;
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
      if (j * 64 < nvec) {   // (uniform)
        const int q = j * 64 + lane;
        const uint32_t word[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int i = 0; i < SPV; ++i) {
          uint32_t sc = 0;
#pragma unroll
          for (int w = 0; w < W; ++w)
#pragma unroll
            for (int g = 0; g < G; ++g) sc += __popc(word[i * W + w] ^ qc[g][w]);
          bool ok = q < nvec;
          if constexpr (PROTECT) ok = ok && pp[j][i] >= a.n_sink && pp[j][i] <= newest_evictable;
          const uint32_t key = ok ? make_key(sc, (uint32_t)(q * SPV + i)) : 0u;
          best = best > key ? best : key;
        }
      }
    }
    return best;
  }

  __device__ __forceinline__ int finish(const DecodeArgs &a, int u, int nv, int t, int lane,
                                        uint32_t *s_code, int *s_e, float *s_vl) {
    const int C = a.C;
    const bool scoring = nv == C || a.scores_dbg != nullptr;
    const bool masked = (a.n_sink | a.n_recent) != 0;
    const bool l2 = W == 1 && a.policy == LSHE_POLICY_L2NORM;
    hash.finish(a, u, lane, s_code);

    int e = nv;
    if (nv == C && !l2 && a.scores_dbg == nullptr) {
      // The common case: every microsecond sooner that the slot is known is a chunk fewer that
      // each streaming wave takes blind (stamps: slot published 4.0 us into the kernel instead
      // of 9.8 us without protected tokens, 5.7 instead of 9.9 us with them).
      uint32_t best = masked ? compact_scan<true>(a, t, lane, s_code) : compact_scan<false>(a, t, lane, s_code);
      best = wave_max_u32(best);
      e = best != 0u ? key_slot(best) : -1;
    } else if (scoring) {
      uint32_t qc[G][W];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int w = 0; w < W; ++w) qc[g][w] = s_code[g * W + w];
      const int newest_evictable = t - 1 - a.n_recent;
      uint32_t best = 0, hi = 0, lo = 0;
#pragma unroll
      for (int j = 0; j < MAXV; ++j) {
        const int q = j * 64 + lane;
        const uint32_t word[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int i = 0; i < SPV; ++i) {
          const int slot = q * SPV + i;
          if (slot < nv) {
            const bool ok = !masked || (pp[j][i] >= a.n_sink && pp[j][i] <= newest_evictable);
            if (l2) {
              const uint32_t c = word[i];
              if (a.scores_dbg) a.scores_dbg[(size_t)u * C + slot] = (int32_t)c;
              const uint32_t h = ok ? c + 1u : 0u;
              if (h > hi) { hi = h; lo = 0xFFFFFu - (uint32_t)slot; }   // ascending slots per lane
            } else {
              uint32_t sc = 0;
#pragma unroll
              for (int w = 0; w < W; ++w)
#pragma unroll
                for (int g = 0; g < G; ++g) sc += __popc(word[i * W + w] ^ qc[g][w]);
              if (a.scores_dbg) a.scores_dbg[(size_t)u * C + slot] = (int32_t)sc;
              const uint32_t key = ok ? make_key(sc, (uint32_t)slot) : 0u;
              best = best > key ? best : key;
            }
          } else if (slot < C && a.scores_dbg) {
            a.scores_dbg[(size_t)u * C + slot] = -1;
          }
        }
      }
      if (nv == C) {
        if (l2) {
          const uint32_t whi = wave_max_u32(hi);
          const uint32_t wlo = wave_max_u32(hi == whi ? lo : 0u);
          e = whi != 0u ? (int)(0xFFFFFu - wlo) : -1;
        } else {
          best = wave_max_u32(best);
          e = best != 0u ? key_slot(best) : -1;
        }
      }
    }
    if (lane == 0 && !a.withhold_victim)
      __hip_atomic_store(s_e, e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);

    if (a.evicted_mass) victim_logits<HD, BF16>(a, u, e, nv == C && e >= 0, lane, s_vl);

    // Algorithm 1 steps 2-5 by the lanes of this wave
    constexpr int VEC = HD * ES / 16;   // 16-byte pieces per row (<= 32)
    if (e >= 0) {
      if (lane < VEC)
        ((uint4 *)((char *)a.K + ((size_t)u * C + e) * HD * ES))[lane] =
            ((const uint4 *)((const char *)a.k_new + (size_t)u * HD * ES))[lane];
      else if (lane >= 32 && lane < 32 + VEC)
        ((uint4 *)((char *)a.V + ((size_t)u * C + e) * HD * ES))[lane - 32] =
            ((const uint4 *)((const char *)a.v_new + (size_t)u * HD * ES))[lane - 32];
      if (lane < W) a.code[((size_t)u * C + e) * W + lane] = s_code[G * W + lane];
      if (lane == W) {
        a.slot_pos[(size_t)u * C + e] = t;
        if (nv < C) a.n_valid[u] = nv + 1;
      }
    }
    if (lane == W + 1 && a.evicted) a.evicted[u] = e;
    return e;
  }
};

template <int HD, int G, int W, bool BF16, int NW, int D>
__global__ __launch_bounds__(64 * NW) void decode_fused_solo_kernel(const DecodeArgs a) {
  constexpr int ES = BF16 ? 2 : 4;
  typedef AttnCore<HD, G, BF16, NW, D, true> Core;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;

  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];
  __shared__ uint32_t s_next;          // next chunk of the K/V stream to hand out
  __shared__ int s_e;                  // the slot written this step, once known
  __shared__ int s_nv;                 // occupied slots before the step (wave 0's read of n_valid)
  __shared__ int s_log[NW][kLogCap];   // chunks a wave consumed before it knew
  __shared__ float s_vl[kMaxGroup];
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ __align__(16) float sm_o[NW][G][HD];

  // Every wave puts its first requests out before the barrier below: wave 0 those of the
  // select, the others their slices of the step inputs and the first chunks of the stream
  // (any row below the budget is a valid address; unoccupied rows are masked when consumed).
  SoloSelect<HD, G, W, BF16> sel;
  Core core;
  Raw8<BF16> ksub, vsub;   // the lane's slices of the new key and value: they stand in for
                           // the written slot in the stream
  auto start_stream = [&]() __attribute__((always_inline)) {
    core.init(a, u, tid, 0, u);
    ksub.load((const char *)a.k_new + ((size_t)u * HD + core.c * 8) * ES);
    vsub.load((const char *)a.v_new + ((size_t)u * HD + core.c * 8) * ES);
    core.prime(a.C);
  };
  // Only wave 0 reads n_valid[u] from memory -- it is also the wave that rewrites it after the
  // select, in program order after its own read -- and hands the value to the other waves
  // through LDS before the barrier, so no wave's read of the count can meet wave 0's write.
  // While the cache is filling the slot to write is simply the next free one.
  // (the two roles meet at one barrier, written once per branch so that the select's
  // registers and the stream's are never live together)
  int nv, e_now;
  if (wave == 0) {
    // The sooner the victim is known, the fewer chunks the streaming waves consume blind and
    // have to read again: the selecting wave goes ahead of the streaming wave it shares a SIMD
    // with (measured: 0.2-0.45 us of a 44 us step; delaying the streaming waves' first loads
    // by 0.2-0.4 us so that the code table's loads meet an idle memory system gains about as
    // much on some boxes and nothing on others, 0.8 us and more loses).
    __builtin_amdgcn_s_setprio(3);
    nv = a.n_valid[u];
    const int t = a.pos[u / a.units_per_seq];
    e_now = nv < a.C ? nv : kVictimUnknown;
    sel.issue(a, u, lane);
    if (lane == 0) { s_next = Core::FIRST_DRAW; s_e = e_now; s_nv = nv; }
    lds_barrier();
    e_now = sel.finish(a, u, nv, t, lane, s_code, &s_e, s_vl);
    __builtin_amdgcn_s_setprio(0);
    start_stream();
  } else {
    start_stream();
    lds_barrier();
    nv = s_nv;
    e_now = nv < a.C ? nv : kVictimUnknown;
  }
  // a full cache stays full; a filling one gains the new token's row
  const int r1 = nv < a.C ? nv + 1 : nv;
  core.stream_deferred(r1, e_now, ksub, vsub, &s_next, &s_e, s_log[wave], a.spin_limit, a.status);
  core.finish(a, u, tid, true, nullptr, a.evicted_mass ? s_vl : nullptr, sm_m, sm_l, sm_o);
}

// ============================================================================================
// host side
// ============================================================================================

// Waves per workgroup of the fused kernel.  With about one unit per CU a big workgroup
// gives the CU enough loads in flight on its own; with many units per CU smaller workgroups
// let one unit's select phase overlap the streaming of its neighbours.
constexpr int kFusedWavesFewUnits = 8, kFusedWavesManyUnits = 4;
// Register stages of the K/V stream: a lone workgroup per CU has registers to spare and needs
// the extra loads in flight; with many workgroups per CU occupancy provides them.
constexpr int kFusedStagesFewUnits = 2, kFusedStagesManyUnits = 2;

template <int HD, bool BF16>
static int launch_select(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const unsigned units = (unsigned)m.units;
  const bool big = m.C > kSelectSmallBudget;
  if (m.W == 1) {
    if (big) hipLaunchKernelGGL((select_kernel<HD, 1, BF16, 1024>), dim3(units), dim3(1024), 0, st, a);
    else hipLaunchKernelGGL((select_kernel<HD, 1, BF16, 256>), dim3(units), dim3(256), 0, st, a);
  } else {
    if (big) hipLaunchKernelGGL((select_kernel<HD, 2, BF16, 1024>), dim3(units), dim3(1024), 0, st, a);
    else hipLaunchKernelGGL((select_kernel<HD, 2, BF16, 256>), dim3(units), dim3(256), 0, st, a);
  }
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
    case 8: {   // two workgroups per (unit, split), 4 query heads each
      const dim3 grid2((unsigned)m.units * (unsigned)a.S * 2u);
      hipLaunchKernelGGL((attn_kernel<HD, 4, BF16>), grid2, block, 0, st, a);
      break;
    }
    default: return LSHE_UNSUPPORTED;
  }
  LSHE_HIP_TRY(hipGetLastError());
  if (a.S > 1) {
    const dim3 cgrid((unsigned)(m.units * m.G)), cblock(kCombineThreads);
    hipLaunchKernelGGL((combine_kernel<HD, BF16>), cgrid, cblock, (size_t)a.S * sizeof(float), st, a);
    LSHE_HIP_TRY(hipGetLastError());
  }
  return LSHE_OK;
}

template <int HD, int G, bool BF16, int NW, int D>
static int launch_fused_solo(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const dim3 grid((unsigned)m.units), block(64 * NW);
  if (m.W == 1)
    hipLaunchKernelGGL((decode_fused_solo_kernel<HD, G, 1, BF16, NW, D>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((decode_fused_solo_kernel<HD, G, 2, BF16, NW, D>), grid, block, 0, st, a);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

template <int HD, int G, bool BF16, int NW, int D>
static int launch_fused_w(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const dim3 grid((unsigned)m.units), block(64 * NW);
  if (m.W == 1)
    hipLaunchKernelGGL((decode_fused_kernel<HD, G, 1, BF16, NW, D>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((decode_fused_kernel<HD, G, 2, BF16, NW, D>), grid, block, 0, st, a);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

template <int HD, int G, bool BF16>
static int launch_fused_g(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  // (the compile-time condition only keeps the 8-wave kernels of heavier heads from being built)
  if constexpr (HD == 128 && G * (BF16 ? 1 : 2) <= 4) {
    if (fused_has_8_waves(m)) {
      // vector loads of the code table and the positions need the arrays 16-byte aligned
      const bool aligned = (((uintptr_t)a.code | (uintptr_t)a.slot_pos) & 15u) == 0;
      if (fused_select_is_solo(m) && aligned)
        return launch_fused_solo<HD, G, BF16, kFusedWavesFewUnits, kFusedStagesFewUnits>(m, a, st);
      return launch_fused_w<HD, G, BF16, kFusedWavesFewUnits, kFusedStagesFewUnits>(m, a, st);
    }
  }
  return launch_fused_w<HD, G, BF16, kFusedWavesManyUnits, kFusedStagesManyUnits>(m, a, st);
}

template <int HD, bool BF16>
static int launch_fused(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  switch (m.G) {
    case 1: return launch_fused_g<HD, 1, BF16>(m, a, st);
    case 2: return launch_fused_g<HD, 2, BF16>(m, a, st);
    case 4: return launch_fused_g<HD, 4, BF16>(m, a, st);
    case 8: return launch_fused_g<HD, 8, BF16>(m, a, st);
    default: return LSHE_UNSUPPORTED;
  }
}

enum { kPhaseSelect = 1, kPhaseAttend = 2 };

#define LSHE_DISPATCH(fn)                                                          \
  (m.d == 128 ? (bf ? fn<128, true>(m, a, st) : fn<128, false>(m, a, st))         \
   : m.d == 64 ? (bf ? fn<64, true>(m, a, st) : fn<64, false>(m, a, st))          \
               : (int)LSHE_UNSUPPORTED)

template <int HD, bool BF16>
static int launch_local(const Dims &m, const DecodeArgs &a, hipStream_t st) {
  const dim3 grid((unsigned)m.units * (unsigned)a.S), block(kAttnThreads);
#define LSHE_AL_CASE(G_)                                                                         \
  case G_:                                                                                        \
    if (m.W == 1) hipLaunchKernelGGL((attn_local_kernel<HD, G_, 1, BF16>), grid, block, 0, st, a); \
    else hipLaunchKernelGGL((attn_local_kernel<HD, G_, 2, BF16>), grid, block, 0, st, a);        \
    break;
  switch (m.G) {
    LSHE_AL_CASE(1)
    LSHE_AL_CASE(2)
    LSHE_AL_CASE(4)
    case 8: {   // two workgroups per (unit, range), 4 query heads each
      const dim3 grid2((unsigned)m.units * (unsigned)a.S * 2u);
      if (m.W == 1) hipLaunchKernelGGL((attn_local_kernel<HD, 4, 1, BF16>), grid2, block, 0, st, a);
      else hipLaunchKernelGGL((attn_local_kernel<HD, 4, 2, BF16>), grid2, block, 0, st, a);
      break;
    }
    default: return LSHE_UNSUPPORTED;
  }
#undef LSHE_AL_CASE
  LSHE_HIP_TRY(hipGetLastError());
  const dim3 cgrid((unsigned)(m.units * m.G));
  if (a.S <= kMergeSmallRanges)
    hipLaunchKernelGGL((merge_small_kernel<HD, BF16>), cgrid, dim3(HD), 0, st, a);
  else
    hipLaunchKernelGGL((merge_local_kernel<HD, BF16>), cgrid, dim3(kCombineThreads), 0, st, a);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}


static int run_phases(const Dims &m, const DecodeArgs &a, int phases, hipStream_t st) {
  const bool bf = m.dtype == LSHE_BF16;
  if (phases == (kPhaseSelect | kPhaseAttend) && decode_is_fused(m.units, m.C, m.G)) return LSHE_DISPATCH(launch_fused);
  // a step asked for whole with several slot ranges per unit: local selects inside the attention
  // kernel, the merge kernel resolves the victim and applies the update (two launches)
  if (phases == (kPhaseSelect | kPhaseAttend) && a.S > 1) return LSHE_DISPATCH(launch_local);
  int rc = LSHE_OK;
  if (phases & kPhaseSelect) {
    rc = LSHE_DISPATCH(launch_select);
    if (rc != LSHE_OK) return rc;
  }
  if (phases & kPhaseAttend) rc = LSHE_DISPATCH(launch_attend);
  return rc;
}

// ---- the select over a code table stored at ONE BYTE PER HASH BIT ---------------------------------
// The paper's implementation keeps every hash bit in a byte (Sections 4.6, 4.7); this build packs
// 32 bits a word.  To put a measured number on what the packing saves, this kernel runs the same
// select -- hash the step inputs, summed Hamming distance to every occupied slot, argmax with
// ties to the lowest slot, kept first / recent tokens -- over a byte table [C][32 W] (byte j of a
// slot = bit j of its code, 0 or 1; bytes >= r are 0), and overwrites the victim's bytes and
// position.  A thread packs a slot's bytes back into words with one multiply per eight bytes
// and then scores as the packed kernel does, so the difference measured is the table's traffic.
template <int HD, int W, bool BF16, int NT>
__global__ __launch_bounds__(NT) void select_unpacked_kernel(const DecodeArgs a, uint8_t *code_bytes) {
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NWAVES = NT / 64, RB = 32 * W;   // bytes per slot
  __shared__ uint32_t s_code[(kMaxGroup + 1) * 2];
  __shared__ uint32_t s_best[NWAVES];
  const int C = a.C, G = a.G;
  const int nv = a.n_valid[u];
  const int t = a.pos[u / a.units_per_seq];
  uint8_t *tab = code_bytes + (size_t)u * C * RB;
  const int32_t *spos = a.slot_pos + (size_t)u * C;
  if (tid < 64) hash_step_inputs<HD, W, BF16>(a, u, tid, s_code);
  lds_barrier();
  const bool masked = (a.n_sink | a.n_recent) != 0;
  const int newest_evictable = t - 1 - a.n_recent;
  uint32_t best = 0;
  for (int s0 = tid; s0 < nv; s0 += 4 * NT) {
    uint4 raw[4][RB / 16];
    int p[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int s = s0 + b * NT < nv ? s0 + b * NT : 0;
#pragma unroll
      for (int k = 0; k < RB / 16; ++k) raw[b][k] = ((const uint4 *)(tab + (size_t)s * RB))[k];
      p[b] = masked ? spos[s] : 0;
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int s = s0 + b * NT;
      if (s < nv) {
        uint32_t sc = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
          // eight bytes of 0/1 -> eight bits: the multiply gathers byte j's bit 0 at bit 56 + j
          const uint4 lo = raw[b][2 * w], hi = raw[b][2 * w + 1];
          const uint64_t q0 = ((uint64_t)lo.y << 32) | lo.x, q1 = ((uint64_t)lo.w << 32) | lo.z;
          const uint64_t q2 = ((uint64_t)hi.y << 32) | hi.x, q3 = ((uint64_t)hi.w << 32) | hi.z;
          constexpr uint64_t M = 0x0102040810204080ull;
          const uint32_t c = (uint32_t)((q0 * M) >> 56) | ((uint32_t)((q1 * M) >> 56) << 8) |
                             ((uint32_t)((q2 * M) >> 56) << 16) | ((uint32_t)((q3 * M) >> 56) << 24);
          for (int g = 0; g < G; ++g) sc += __popc(c ^ s_code[g * W + w]);
        }
        const bool ok = !masked || (p[b] >= a.n_sink && p[b] <= newest_evictable);
        const uint32_t key = ok ? make_key(sc, (uint32_t)s) : 0u;
        best = best > key ? best : key;
      }
    }
  }
  best = wave_max_u32(best);
  if (lane == 0) s_best[wave] = best;
  lds_barrier();
#pragma unroll
  for (int k = 0; k < NWAVES; ++k) best = best > s_best[k] ? best : s_best[k];
  const int e = nv < C ? nv : (best != 0u ? key_slot(best) : -1);
  if (e >= 0) {
    if (tid < RB) tab[(size_t)e * RB + tid] = (uint8_t)((s_code[G * W + tid / 32] >> (tid & 31)) & 1u);
    if (tid == 64) {
      a.slot_pos[(size_t)u * C + e] = t;
      if (nv < C) a.n_valid[u] = nv + 1;
    }
  }
  if (tid == 65 && a.evicted) a.evicted[u] = e;
}

// ---- scratch memory of the library's own, for callers that cannot allocate -------------------
// A file-scope device array takes the place of the `workspace` argument (partial softmax states,
// the victim's logits, the select's hand-over to the merge kernel).  Every GPU holds its own copy
// of the array at its own address, looked up once per device with hipGetSymbolAddress while that
// device is current; host code only ever passes the looked-up pointer to kernels, never the
// array's name.  Nothing in it has to start at zero (every word a step reads was written earlier
// in the same step), so there is nothing to clear between calls.
constexpr size_t kBuiltinScratchBytes = LSHE_BUILTIN_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kBuiltinScratchBytes];
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static int builtin_scratch_ptr(void **out) {
  int dev = -1;
  LSHE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return LSHE_HIP_ERROR;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    LSHE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255u) != 0) return LSHE_HIP_ERROR;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LSHE_OK;
}

// Polls (of about 0.3 us each) a streaming wave makes for the victim's slot before it gives up:
// several seconds, against a wait that lasts some microseconds when all is well.
constexpr int kSpinLimitDefault = 1 << 24;
static std::atomic<int> g_spin_limit{kSpinLimitDefault};
static std::atomic<int> g_withhold_victim{0};

// Argument checks and DecodeArgs shared by the entry points; pointers a phase does not
// use may be NULL for that phase.
static int decode_common(const lshe_config *cfg, const void *R_dev, const void *q_new,
                         const void *k_new, const void *v_new, const int32_t *pos, void *K_cache,
                         void *V_cache, uint32_t *code_cache, int32_t *slot_pos, int32_t *n_valid,
                         void *out, int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                         float *evicted_mass, void *workspace, size_t workspace_bytes, void *stream,
                         int phases, bool builtin_scratch = false) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (builtin_scratch) {
    // the library's own scratch array stands in for the caller's workspace: checked against
    // what the plan of this configuration really touches (the single-kernel plans: nothing)
    const Dims m0 = dims_of(cfg);
    // (the status word alone for the single-kernel plans)
    const size_t need = decode_is_fused(m0.units, m0.C, m0.G) ? kWsHeaderBytes : decode_ws_bytes(m0);
    if (need > kBuiltinScratchBytes) return LSHE_SCRATCH_EXCEEDED;
    rc = builtin_scratch_ptr(&workspace);
    if (rc != LSHE_OK) return rc;
    workspace_bytes = decode_ws_bytes(m0);   // (checked against the plan's real need above)
  }
  if (!q_new || !K_cache || !V_cache || !n_valid || !workspace) return LSHE_INVALID_ARG;
  if ((phases & kPhaseSelect) && (!k_new || !v_new || !pos || !code_cache || !slot_pos))
    return LSHE_INVALID_ARG;
  if ((phases & kPhaseSelect) && !R_dev && cfg->policy != LSHE_POLICY_L2NORM) return LSHE_INVALID_ARG;
  if ((phases & kPhaseAttend) && !out) return LSHE_INVALID_ARG;
  const Dims m = dims_of(cfg);
  if (m.G != 1 && m.G != 2 && m.G != 4 && m.G != 8) return LSHE_UNSUPPORTED;
  if (workspace_bytes < decode_ws_bytes(m)) return LSHE_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)workspace & 255u) != 0) return LSHE_INVALID_ARG;

  DecodeArgs a;
  a.R_dev = R_dev; a.q = q_new; a.k_new = k_new; a.v_new = v_new; a.pos = pos;
  a.K = K_cache; a.V = V_cache; a.code = code_cache; a.slot_pos = slot_pos; a.n_valid = n_valid;
  a.out = out; a.evicted = evicted; a.scores_dbg = scores_dbg; a.codes_dbg = codes_dbg;
  a.status = (int32_t *)workspace;
  a.partials = (float *)((char *)workspace + kWsHeaderBytes);
  a.victim_logit = (float *)((char *)a.partials + decode_ws_partial_bytes(m));
  a.sel_out = (int32_t *)((char *)a.victim_logit + decode_ws_logit_bytes(m));
  a.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
  a.withhold_victim = g_withhold_victim.load(std::memory_order_relaxed);
  a.evicted_mass = phases == (kPhaseSelect | kPhaseAttend) ? evicted_mass : nullptr;
  a.C = m.C; a.G = m.G; a.r = m.r; a.units_per_seq = m.L * m.H;
  a.n_sink = m.n_sink; a.n_recent = m.n_recent; a.policy = m.policy;
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
                                int32_t *scores_dbg, uint32_t *codes_dbg, float *evicted_mass,
                                void *workspace, size_t workspace_bytes, void *stream) {
  return decode_common(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                       n_valid, out, evicted, scores_dbg, codes_dbg, evicted_mass, workspace,
                       workspace_bytes, stream, kPhaseSelect | kPhaseAttend);
}

extern "C" int lshe_decode_select(const lshe_config *cfg, const void *R_dev, const void *q_new,
                                  const void *k_new, const void *v_new, const int32_t *pos,
                                  void *K_cache, void *V_cache, uint32_t *code_cache,
                                  int32_t *slot_pos, int32_t *n_valid, int32_t *evicted,
                                  int32_t *scores_dbg, uint32_t *codes_dbg, void *workspace,
                                  size_t workspace_bytes, void *stream) {
  return decode_common(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                       n_valid, nullptr, evicted, scores_dbg, codes_dbg, nullptr, workspace,
                       workspace_bytes, stream, kPhaseSelect);
}

extern "C" int lshe_decode_attend(const lshe_config *cfg, const void *q_new, const void *K_cache,
                                  const void *V_cache, const int32_t *n_valid, void *out,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  return decode_common(cfg, nullptr, q_new, nullptr, nullptr, nullptr, (void *)K_cache,
                       (void *)V_cache, nullptr, nullptr, (int32_t *)n_valid, out, nullptr, nullptr,
                       nullptr, nullptr, workspace, workspace_bytes, stream, kPhaseAttend);
}


extern "C" int lshe_decode_step_noalloc(const lshe_config *cfg, const void *R_dev, const void *q_new,
                                        const void *k_new, const void *v_new, const int32_t *pos,
                                        void *K_cache, void *V_cache, uint32_t *code_cache,
                                        int32_t *slot_pos, int32_t *n_valid, void *out,
                                        int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                                        float *evicted_mass, void *stream) {
  return decode_common(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                       n_valid, out, evicted, scores_dbg, codes_dbg, evicted_mass, nullptr, 0, stream,
                       kPhaseSelect | kPhaseAttend, true);
}

extern "C" void lshe_debug_select_wait(int32_t spin_limit, int32_t withhold_victim) {
  g_spin_limit.store(spin_limit > 0 ? spin_limit : kSpinLimitDefault, std::memory_order_relaxed);
  g_withhold_victim.store(withhold_victim != 0, std::memory_order_relaxed);
}

#ifdef LSHE_STAMPS
// instrumented build only: the decode kernels' stamps, copied to the host / cleared
extern "C" int lshe_read_stamps(unsigned long long *host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(lshe::g_stamps), bytes);
}
extern "C" int lshe_clear_stamps(void) {
  void *p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(lshe::g_stamps)) != hipSuccess) return -1;
  return (int)hipMemset(p, 0, sizeof(lshe::g_stamps));
}
#endif

extern "C" int lshe_decode_select_unpacked(const lshe_config *cfg, const void *R_dev, const void *q_new,
                                           const void *k_new, const int32_t *pos, uint8_t *code_bytes,
                                           int32_t *slot_pos, int32_t *n_valid, int32_t *evicted,
                                           void *stream) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (!R_dev || !q_new || !k_new || !pos || !code_bytes || !slot_pos || !n_valid) return LSHE_INVALID_ARG;
  if (cfg->policy != LSHE_POLICY_HASH) return LSHE_UNSUPPORTED;
  const Dims m = dims_of(cfg);
  if (m.G != 1 && m.G != 2 && m.G != 4 && m.G != 8) return LSHE_UNSUPPORTED;
  if (m.d != 128 || m.dtype != LSHE_BF16) return LSHE_UNSUPPORTED;   // the measured configurations only
  DecodeArgs a = {};
  a.R_dev = R_dev; a.q = q_new; a.k_new = k_new; a.pos = pos;
  a.slot_pos = slot_pos; a.n_valid = n_valid; a.evicted = evicted;
  a.C = m.C; a.G = m.G; a.r = m.r; a.units_per_seq = m.L * m.H;
  a.n_sink = m.n_sink; a.n_recent = m.n_recent; a.policy = m.policy;
  const dim3 grid((unsigned)m.units), block(256);
  if (m.W == 1) hipLaunchKernelGGL((select_unpacked_kernel<128, 1, true, 256>), grid, block, 0, (hipStream_t)stream, a, code_bytes);
  else hipLaunchKernelGGL((select_unpacked_kernel<128, 2, true, 256>), grid, block, 0, (hipStream_t)stream, a, code_bytes);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}
