// lshe_prefill_compress: the Prompt Encoding Stage of Section 3.
//
//   1. hash every prompt key, and every query of tokens >= C, on the matrix cores (eq. 2);
//   2. run Algorithm 1 steps 1-5 token by token on the CODE TABLE ALONE: the eviction
//      decision (eq. 5-6) reads only hash codes, never K/V values, so the sequential part
//      touches C*W words per unit, held in LDS; the scores of 32 steps at a time come from
//      an i8 matrix product on the matrix cores (evict_mfma_kernel), or from XOR + popcount
//      in bit-sliced form in the vector ALU (evict_lds_kernel: narrow hashes, small budgets);
//   3. gather the surviving tokens' K, V and codes into the slot arrays once.
// The result is the same as inserting the tokens one at a time.
#include <atomic>
#include <mutex>

#include "lshe_kernels.h"

namespace lshe {

// Counters and wall-clock totals of an instrumented build (-DLSHE_STAMPS); compiled out otherwise.
#ifdef LSHE_STAMPS
#define LSHE_STAT(...) __VA_ARGS__
#else
#define LSHE_STAT(...)
#endif

struct EvictArgs {
  const uint32_t *codes_k;   // [units][N][W]
  const uint32_t *codes_q;   // [units][G][N-C][W]
  uint32_t *code_cache;      // [units][C][W]   (used by the large-budget kernel only)
  int32_t *slot_pos;         // [units][C]
  int32_t *n_valid;          // [units]
  int32_t *evict_log;        // nullable [units][N-C]
  int C, G, N, n_sink, n_recent;
  long long units;
  int t_begin, t_end;        // evict_mfma_kernel: the tokens [t_begin, t_end) of this launch (C and N for
                             // the whole prompt stage in one launch; a later launch takes the table up
                             // from code_cache and slot_pos, where the one before it left it)
};

// ---- bit-sliced score -----------------------------------------------------------------------
// For hash bit b let n_b = number of the G query codes with bit b set.  A cached code c
// contributes (c_b ? G - n_b : n_b) to the summed Hamming distance.  Written in binary,
// plane p of that contribution is c_b on the bits where plane p of n_b is 0 and of G - n_b
// is 1 (mask A_p), NOT c_b where it is the other way round (mask B_p), and a constant
// elsewhere.  Hence
//     score(c) = const + sum_p 2^p * popcount((c & A_p) | (~c & B_p)),
// one bit-field-insert and one popcount per plane and word instead of one XOR and one
// popcount per query head and word.  For even G plane 0 is constant, so the planes that
// matter are 1..log2(G): NP = 1, 1, 2, 3 planes for G = 1, 2, 4, 8.  Ordering and ties of
// the reduced score equal those of the exact one.
template <int W, int NP>
struct Planes {
  uint32_t A[NP][W], B[NP][W];
};

// x: the G query codes of this step (wave-uniform values); P0: first plane that varies
template <int W, int NP, int GMAX>
__device__ __forceinline__ void make_planes(const uint32_t (&x)[GMAX][W], int G, int P0,
                                            Planes<W, NP> &pl) {
#pragma unroll
  for (int w = 0; w < W; ++w) {
    uint32_t n[4] = {0, 0, 0, 0}, z[4] = {0, 0, 0, 0};   // bit-sliced counts of ones / zeros
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
      if (g < G) {
        uint32_t carry = x[g][w];
#pragma unroll
        for (int p = 0; p < 4; ++p) { const uint32_t t = n[p] & carry; n[p] ^= carry; carry = t; }
        carry = ~x[g][w];
#pragma unroll
        for (int p = 0; p < 4; ++p) { const uint32_t t = z[p] & carry; z[p] ^= carry; carry = t; }
      }
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      uint32_t np = 0, zp = 0;
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p == P0 + i) { np = n[p]; zp = z[p]; }
      pl.A[i][w] = ~np & zp;
      pl.B[i][w] = np & ~zp;
    }
  }
}

template <int W, int NP>
__device__ __forceinline__ uint32_t plane_score(const uint32_t (&c)[W], const Planes<W, NP> &pl) {
  uint32_t sc = 0;
#pragma unroll
  for (int i = NP - 1; i >= 0; --i) {
    uint32_t a = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) a += __popc((c[w] & pl.A[i][w]) | (~c[w] & pl.B[i][w]));
    sc = (sc << 1) + a;
  }
  return sc;
}

// ---- sequential eviction with the code table in LDS ------------------------------------------
// One workgroup of NT = 64*WAVES threads per unit; LDS holds tab[C][W] (and pos[C] when some
// tokens are protected).  Thread `tid` owns slots tid, tid + NT, ...: it is the only reader
// and writer of those entries, so the table needs no barrier; consecutive lanes touch
// consecutive words (no bank conflicts).  Bits of codes beyond r are zero in keys and queries
// alike, so they never score.  The codes of the next 64 tokens (G query codes + key code
// each) are fetched one chunk ahead, one token per lane, turned into plane masks for all 64
// tokens at once, and handed to the step loop with v_readlane, so no step waits on global
// memory or spends scalar work on its query codes.
template <int W>
struct CodeWords;
template <>
struct CodeWords<1> {
  uint32_t c[1];
  __device__ __forceinline__ void load(const uint32_t *p) { c[0] = p[0]; }
};
template <>
struct CodeWords<2> {
  uint32_t c[2];
  __device__ __forceinline__ void load(const uint32_t *p) {
    const uint2 v = *(const uint2 *)p;
    c[0] = v.x; c[1] = v.y;
  }
};

template <int W, int NP, bool MASKED, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void evict_lds_kernel(const EvictArgs a, int P0) {
  constexpr int NT = 64 * WAVES;
  constexpr int GMAX = NP == 1 ? 2 : NP == 2 ? 4 : 8;
  constexpr int UNR = 4;
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int C = a.C, N = a.N, G = a.G, NQ = N - C;
  const uint32_t *ck = a.codes_k + (size_t)u * N * W;
  const uint32_t *cq = a.codes_q + (size_t)u * G * NQ * W;
  int32_t *spos = a.slot_pos + (size_t)u * C;

  extern __shared__ __align__(16) uint32_t lds[];
  uint32_t *tab = lds;                                   // [C][W]
  int32_t *pos = (int32_t *)(lds + (size_t)C * W);       // [C]      (MASKED only)
  uint32_t *s_best = lds + (size_t)C * W + (MASKED ? C : 0) + (((size_t)C * W + (MASKED ? C : 0)) & 1);

  for (int s = tid; s < C; s += NT) {
#pragma unroll
    for (int w = 0; w < W; ++w) tab[(size_t)s * W + w] = ck[(size_t)s * W + w];
    if constexpr (MASKED) pos[s] = s;
    spos[s] = s;
  }

  uint32_t qn[GMAX][W], kn[W];
  auto fetch = [&](int tb) __attribute__((always_inline)) {   // lane l takes token tb + l
    const int tt = tb + lane;
#pragma unroll
    for (int g = 0; g < GMAX; ++g)
#pragma unroll
      for (int w = 0; w < W; ++w)
        qn[g][w] = (g < G && tt < N) ? cq[((size_t)g * NQ + (tt - C)) * W + w] : 0u;
#pragma unroll
    for (int w = 0; w < W; ++w) kn[w] = tt < N ? ck[(size_t)tt * W + w] : 0u;
  };
  fetch(C);

  const int jfull = C / NT;                  // rows of the table in which every thread has a slot
  const bool has_tail = jfull * NT + tid < C;
  const uint32_t key0 = (1u << 20) + (0xFFFFFu - (uint32_t)tid);   // key of (score 0, slot tid)
  const uint32_t *mytab = tab + (size_t)tid * W;
  const int32_t *mypos = pos + tid;

  for (int tb = C; tb < N; tb += 64) {
    // This chunk's tokens, one per lane: the plane masks of the token's G query codes are
    // computed here in the vector ALU for all 64 tokens at once, so a step only has to
    // read its token's masks and key code out of the lanes.
    Planes<W, NP> plv;
    make_planes<W, NP, GMAX>(qn, G, P0, plv);
    uint32_t kc[W];
#pragma unroll
    for (int w = 0; w < W; ++w) kc[w] = kn[w];
    if (tb + 64 < N) fetch(tb + 64);
    const int tend = tb + 64 < N ? tb + 64 : N;

    for (int t = tb; t < tend; ++t) {
      const int li = t - tb;
      Planes<W, NP> pl;
      uint32_t nk[W];
#pragma unroll
      for (int i = 0; i < NP; ++i)
#pragma unroll
        for (int w = 0; w < W; ++w) {
          pl.A[i][w] = (uint32_t)__builtin_amdgcn_readlane((int)plv.A[i][w], li);
          pl.B[i][w] = (uint32_t)__builtin_amdgcn_readlane((int)plv.B[i][w], li);
        }
#pragma unroll
      for (int w = 0; w < W; ++w) nk[w] = (uint32_t)__builtin_amdgcn_readlane((int)kc[w], li);
      const int newest_evictable = t - 1 - a.n_recent;

      // key = ((score + 1) << 20) | (0xFFFFF - slot), built as (score << 20) + (key0 - j*NT)
      uint32_t best = 0, koff = key0;
      auto visit = [&](const CodeWords<W> &cw, int p) __attribute__((always_inline)) {
        uint32_t key = (plane_score<W, NP>(cw.c, pl) << 20) + koff;
        if constexpr (MASKED) key = (p >= a.n_sink && p <= newest_evictable) ? key : 0u;
        best = best > key ? best : key;
        koff -= NT;
      };
      // rows in groups of UNR, two groups in flight: the LDS reads of the next group are
      // issued before the current group is scored
      CodeWords<W> ga[UNR], gb[UNR];
      int pa[UNR], pb[UNR];
      auto load_group = [&](CodeWords<W> (&cw)[UNR], int (&pp)[UNR], int row) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
          cw[i].load(mytab + (size_t)(row + i) * NT * W);
          pp[i] = MASKED ? mypos[(size_t)(row + i) * NT] : 0;
        }
      };
      auto score_group = [&](const CodeWords<W> (&cw)[UNR], const int (&pp)[UNR]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) visit(cw[i], pp[i]);
      };
      int j = 0;
      if (UNR <= jfull) load_group(ga, pa, 0);
      for (; j + UNR <= jfull; j += 2 * UNR) {
        const bool second = j + 2 * UNR <= jfull;
        if (second) load_group(gb, pb, j + UNR);
        score_group(ga, pa);
        if (second) {
          if (j + 3 * UNR <= jfull) load_group(ga, pa, j + 2 * UNR);
          score_group(gb, pb);
        }
      }
      j = jfull / UNR * UNR;
      for (; j < jfull; ++j) {
        CodeWords<W> cw;
        cw.load(mytab + (size_t)j * NT * W);
        visit(cw, MASKED ? mypos[(size_t)j * NT] : 0);
      }
      if (has_tail) {
        CodeWords<W> cw;
        cw.load(mytab + (size_t)jfull * NT * W);
        visit(cw, MASKED ? mypos[(size_t)jfull * NT] : 0);
      }

      best = wave_max_u32(best);
      if (WAVES > 1) {
        if (lane == 0) s_best[(t & 1) * WAVES + wave] = best;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < WAVES; ++k) {
          const uint32_t o = s_best[(t & 1) * WAVES + k];
          best = best > o ? best : o;
        }
      }
      if (best == 0u) continue;   // no evictable slot (cannot happen for a valid config)
      const int e = key_slot(best);
      if (tid == e % NT) {        // the owner of slot e
#pragma unroll
        for (int w = 0; w < W; ++w) tab[(size_t)e * W + w] = nk[w];
        if constexpr (MASKED) pos[e] = t;
        spos[e] = t;
        if (a.evict_log) a.evict_log[(size_t)u * NQ + (t - C)] = e;
      }
    }
  }
  if (tid == 0) a.n_valid[u] = C;
}

// ---- sequential eviction with the scores taken on the matrix cores ----------------------------
// The summed Hamming distance of a cached code c to the G query codes of a step is
//     sum_b n_b + sum_b c_b * (G - 2 n_b),          n_b = number of query codes with bit b set,
// i.e. up to a per-step constant an inner product of the code's bits with integer weights:
// a matrix product [T steps x r bits] * [r bits x C slots].  The table changes by one slot per
// step, so T = 32 steps are scored at once against the table as it stands at the start of the
// block (v_mfma_i32_32x32x32_i8: 32 slots a tile as rows, the steps as columns, one MFMA per
// code word), each lane keeping a running best for its step over its rows of every tile; then
// one wave walks the 32 steps in order.  For step i the winner is the larger of
//   * the best slot of the unchanged table, which stands unless that very slot was overwritten
//     by an earlier step of the block (all other slots of the old table score no higher), and
//   * the block's own earlier tokens, whose scores against all 32 steps come from one more tile.
// If the old winner was overwritten, the walking wave resolves the step from a short candidate
// list: the table's groups (the 16 slots of a tile that one lane holds) are partitioned by
// (wave, half), and every lane keeps the best TWO group maxima of its partition for its step.
// A candidate group whose best slot has been overwritten (or is a protected recent token) is
// scored again, 16 slots, on the table as it stands; groups outside the lists all lie below the
// second maximum of their partition, so when the best candidate found is no lower than every
// partition's second maximum it is the step's exact argmax.  Only when that test fails (about
// one conflict in a hundred) does every wave score its share of the whole table.  Victims equal
// the step-by-step definition, ties included (lower tile and row, i.e. lower slot, win at
// every stage).
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));
#ifndef LSHE_MFMA_STEPS
#define LSHE_MFMA_STEPS 32
#endif
constexpr int kMfmaSteps = LSHE_MFMA_STEPS;   // steps per block: 32 or 64 (one or two column sets per tile)
constexpr int kMfmaStaleLimit = 10 * (kMfmaSteps / 32);    // of the steps of a block
constexpr int kMfmaDirectBlocks = 12 / (kMfmaSteps / 32);
constexpr int kMfmaMaxTiles = 2048;   // tile number field of the running key

// Bits -> operand bytes.  The MFMA wants one byte per hash bit; which k index a bit gets, and
// with what factor, is free as long as the weights agree.  With t = c >> 4 half, dword m of the
// lane's 16 bytes is t & (0x01010101 << m): byte j holds bit 8 j + m + 4 half of c, worth 2^m,
// and the weights of dword m are scaled by 16 >> m instead of 16 -- every product is still
// 16 (G - 2 n_b) c_b.  One shift and four ANDs per code word instead of three operations per
// four bits.
__device__ __forceinline__ v4i_t spread16(uint32_t c, int half) {
  const uint32_t t = c >> (4 * half);
  v4i_t r;
#pragma unroll
  for (int m = 0; m < 4; ++m) r[m] = (int)(t & (0x01010101u << m));
  return r;
}

// Blocks of 64 steps (kMfmaSteps = 64: the bits -> bytes expansion of a tile paid once per two
// column sets of 32 steps, half as many barriers and walks) are supported by this source and
// were measured three times.  Before the walk was made cheap they lost outright (12.4 against
// 11.0 ms on the prefill workload: more registers, three waves per SIMD instead of five, and a
// serial walk twice as long).  With the present walk they gain 4 % on independent queries
// (eviction phase 2.63 against 2.74 ms; 3.6 against 4.7 ms on the 8 units of the long-context
// prompt, which are bound by latency per block) and lose as soon as queries are correlated: a
// block-start table that is 64 steps old has its winners taken twice as often (query correlation
// 0.3 / 0.5 / 0.9: 4.34 / 6.93 / 10.61 against 3.58 / 5.06 / 8.47 ms; with 4 + 10 kept tokens 3.11
// against 2.99 ms; one layer's 8 units at correlation 0.5: 0.86 against 0.67 ms, the long-context
// prompt 11.0 against 9.4 ms).  Real queries are correlated, so blocks stay at 32 steps
// (-DLSHE_MFMA_STEPS=64 builds the other form).
// MASKED (some tokens are never evicted): the first n_sink tokens sit in slots 0 .. n_sink-1 for
// good, so those slots are simply left out of the matrix product; the n_recent newest tokens
// are left in, and a step whose unchanged-table winner turns out to be one of them (rare: a
// handful of C slots, and recent tokens tend to be close to the query) is rescored like a step
// whose winner was overwritten.
template <int W, int WAVES, int GMAX, bool MASKED>
__global__ __launch_bounds__(64 * WAVES)
__attribute__((amdgpu_waves_per_eu((MASKED || GMAX == 8 || kMfmaSteps == 64) ? 4 : 5)))
void evict_mfma_kernel(const EvictArgs a, int P0) {
  constexpr int NT = 64 * WAVES;
  constexpr int T = kMfmaSteps;
  constexpr int NCS = T / 32;    // column sets of a tile: steps 32 cs + col
  constexpr int SNS = T + 2;     // row stride of s_new (16-bit entries)
  static_assert(T == 32 || T == 64, "a block is one or two sets of 32 steps");
  constexpr int NP = GMAX == 2 ? 1 : GMAX == 4 ? 2 : 3;   // planes of the bit-sliced score
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  // (through readfirstlane so that the compiler knows the wave number, and with it the walker's
  // control flow and step counter, to be wave-uniform: scalar branches, counter in an SGPR)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;   // operand row/column of the lane; its k half
  const int C = a.C, N = a.N, G = a.G, NQ = N - C;
  const uint32_t *ck = a.codes_k + (size_t)u * N * W;
  const uint32_t *cq = a.codes_q + (size_t)u * G * NQ * W;
  int32_t *spos = a.slot_pos + (size_t)u * C;

  extern __shared__ __align__(16) uint32_t lds[];
  uint32_t *tab = lds;                               // [C][W]
  int *s_part = (int *)(lds + (size_t)C * W);        // [WAVES][T] per-wave best key per step
  int16_t *s_new = (int16_t *)(s_part + WAVES * T);  // [T steps][T + 2]: tokens of the block (padded row)
  uint32_t *s_flag = (uint32_t *)(s_new + T * SNS);  // [0] the step to rescore, [1 + wave] its keys,
                                                     // [1 + WAVES] blocks to take step by step
  constexpr int NCAND = 4 * WAVES;                   // candidate groups per step: 2 per (wave, half)
  uint32_t *s_cand = s_flag + 2 + WAVES;             // [T][NCAND] keys ((score + 1) << 20 | ~slot) of the candidates
  uint32_t *s_written = (uint32_t *)(s_cand + T * NCAND);   // [(C + 31) / 32] bit per slot: written in this block
  uint32_t *s_seen = s_written + (C + 31) / 32;             // [(C + 31) / 32] scratch bits, zero between uses
  int *s_wt = (int *)(s_seen + (C + 31) / 32);              // [NCS][4 W][64] the next block's weights, see below
  int32_t *pos = (int32_t *)(s_wt + NCS * 4 * W * 64);      // [C] token in each slot (MASKED only)

  const int TE = a.t_end;   // this launch's tokens end here
  uint32_t *saved = a.code_cache + (size_t)u * C * W;   // the table between two launches
  if (a.t_begin == C) {
    for (int s = tid; s < C; s += NT) {
#pragma unroll
      for (int w = 0; w < W; ++w) tab[(size_t)s * W + w] = ck[(size_t)s * W + w];
      if constexpr (MASKED) pos[s] = s;
      spos[s] = s;
    }
  } else {
    for (int s = tid; s < C; s += NT) {
#pragma unroll
      for (int w = 0; w < W; ++w) tab[(size_t)s * W + w] = saved[(size_t)s * W + w];
      if constexpr (MASKED) pos[s] = spos[s];
    }
  }
  for (int k = tid; k < 2 * ((C + 31) / 32); k += NT) s_written[k] = 0u;   // and s_seen behind it
  __syncthreads();

  const int n_tiles = (C + 31) / 32;
  const int bias = G * 32 * W + 1;   // keeps the biased score sum_b c_b (G - 2 n_b) + bias >= 1

  // codes of the block's token t0 + tok: its G query codes and its key code (with 32 steps a
  // block both halves of the wave hold the same token, with 64 every lane its own)
  const int tok = T == 64 ? lane : col;
  uint32_t qn[GMAX][W], kn[W];
  auto fetch = [&](int t0) __attribute__((always_inline)) {
    const int tt = t0 + tok;
#pragma unroll
    for (int g = 0; g < GMAX; ++g)
#pragma unroll
      for (int w = 0; w < W; ++w)
        qn[g][w] = (g < G && tt < TE) ? cq[((size_t)g * NQ + (tt - C)) * W + w] : 0u;
#pragma unroll
    for (int w = 0; w < W; ++w) kn[w] = tt < TE ? ck[(size_t)tt * W + w] : 0u;
  };
  fetch(a.t_begin);

  // Every wave scores its share of the table as it stands for one step (plane masks pl) with
  // the bit-sliced score of evict_lds_kernel; returns the winning key to all threads.  Two
  // barriers; the caller adds the one that orders the slot update.
  auto scan_table = [&](const Planes<W, NP> &pl, int t) __attribute__((always_inline)) {
    uint32_t win = 0;
    const int newest_evictable = t - 1 - a.n_recent;
#pragma unroll 4
    for (int sl = tid; sl < C; sl += NT) {
      CodeWords<W> cw;
      cw.load(tab + (size_t)sl * W);
      uint32_t key = make_key(plane_score<W, NP>(cw.c, pl), (uint32_t)sl);
      if constexpr (MASKED) key = (pos[sl] >= a.n_sink && pos[sl] <= newest_evictable) ? key : 0u;
      win = win > key ? win : key;
    }
    win = wave_max_u32(win);
    if (lane == 0) s_flag[1 + wave] = win;
    __syncthreads();
    win = 0;
#pragma unroll
    for (int k = 0; k < WAVES; ++k) {
      const uint32_t o = s_flag[1 + k];
      win = win > o ? win : o;
    }
    return win;
  };

  LSHE_STAT(unsigned long long st_t0 = 0, st_tiles = 0, st_walk = 0, st_block = 0, st_tb = 0, st_bar = 0, st_pre = 0, st_pa = 0;
            unsigned long long st_pass = 0, st_single = 0, st_conf = 0, st_fall = 0;)
  int turn = u;   // the wave that walks a block's steps alone: a different one every block, so
                  // that the serial work of the units sharing a CU spreads over its four SIMDs
  bool wt_shared = false;   // s_wt holds the weights of the block about to start
  int direct_left = 0;   // blocks still to be taken step by step (see below)
  int direct_run = kMfmaDirectBlocks;   // length of the next such run: doubles while the trial blocks between runs stay bad
  for (int t0 = a.t_begin; t0 < TE; t0 += T, ++turn) {
    const bool walker = wave == turn % WAVES;
    const int n_steps = TE - t0 < T ? TE - t0 : T;
    uint32_t qc[GMAX][W], kc[W];
#pragma unroll
    for (int g = 0; g < GMAX; ++g)
#pragma unroll
      for (int w = 0; w < W; ++w) qc[g][w] = qn[g][w];
#pragma unroll
    for (int w = 0; w < W; ++w) kc[w] = kn[w];
    if (t0 + T < TE) fetch(t0 + T);

    // slot e takes the block's token `step` (one wave calls this)
    auto store_token = [&](int e, int step) __attribute__((always_inline)) {
#pragma unroll
      for (int w = 0; w < W; ++w) {
        const uint32_t nk = (uint32_t)__builtin_amdgcn_readlane((int)kc[w], step);
        if (lane == w) tab[(size_t)e * W + w] = nk;
      }
      if (lane == 0) {
        if constexpr (MASKED) pos[e] = t0 + step;
        spos[e] = t0 + step;
        if (a.evict_log) a.evict_log[(size_t)u * NQ + (t0 + step - C)] = e;
        atomicOr(&s_written[e >> 5], 1u << (e & 31));
      }
    };

    if (direct_left > 0) {
      // ---- a block taken step by step: the vector-ALU kernel's step, 32 times -----------------
      --direct_left;
      Planes<W, NP> plv;   // lane col: plane masks of step col
      make_planes<W, NP, GMAX>(qc, G, P0, plv);
      for (int i = 0; i < n_steps; ++i) {
        Planes<W, NP> pl;
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int w = 0; w < W; ++w) {
            pl.A[p][w] = (uint32_t)__builtin_amdgcn_readlane((int)plv.A[p][w], i);
            pl.B[p][w] = (uint32_t)__builtin_amdgcn_readlane((int)plv.B[p][w], i);
          }
        // One barrier per step, as in the vector-ALU kernel: thread tid is the only reader of
        // slots tid, tid + NT, ... here, so the thread that owns the winning slot writes the new
        // code itself, and the waves' partial maxima alternate between two rows of s_part (a
        // wave can be a step ahead of one still reading the previous row, never two).
        uint32_t win = 0;
        const int newest_evictable = t0 + i - 1 - a.n_recent;
#pragma unroll 4
        for (int sl = tid; sl < C; sl += NT) {
          CodeWords<W> cw;
          cw.load(tab + (size_t)sl * W);
          uint32_t key = make_key(plane_score<W, NP>(cw.c, pl), (uint32_t)sl);
          if constexpr (MASKED) key = (pos[sl] >= a.n_sink && pos[sl] <= newest_evictable) ? key : 0u;
          win = win > key ? win : key;
        }
        win = wave_max_u32(win);
        int *row = s_part + (i & 1) * WAVES;
        if (lane == 0) row[wave] = (int)win;
        __syncthreads();
        win = 0;
#pragma unroll
        for (int k = 0; k < WAVES; ++k) {
          const uint32_t o = (uint32_t)row[k];
          win = win > o ? win : o;
        }
        if (win != 0u) {
          const int e = key_slot(win);
#pragma unroll
          for (int w = 0; w < W; ++w) {
            const uint32_t nk = (uint32_t)__builtin_amdgcn_readlane((int)kc[w], i);
            if (tid == e % NT) tab[(size_t)e * W + w] = nk;
          }
          if (tid == e % NT) {
            if constexpr (MASKED) pos[e] = t0 + i;
            spos[e] = t0 + i;
            if (a.evict_log) a.evict_log[(size_t)u * NQ + (t0 + i - C)] = e;
          }
        }
      }
      __syncthreads();   // the next block's matrix product reads every slot from every wave
      wt_shared = false;
      continue;
    }

    LSHE_STAT(st_t0 = __builtin_amdgcn_s_memrealtime(); st_tb = st_t0;)
    // weights (16 >> m) (G - 2 n_b) of step `col` for the bits of dword m of spread16, as signed
    // bytes (|.| <= 64); the factor 16 on a product leaves its low 4 bits for the
    // slot's rank inside the lane (below)
    auto make_weights = [&](const uint32_t (&qx)[GMAX][W], v4i_t (&out)[W]) __attribute__((always_inline)) {
#pragma unroll
      for (int w = 0; w < W; ++w)
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          uint32_t n = 0;   // per byte: how many of the G codes have the bit (heads >= G are zero)
#pragma unroll
          for (int g = 0; g < GMAX; ++g) n += (qx[g][w] >> (4 * half + m)) & 0x01010101u;
          // bytewise s G - 2 s n, s = 16 >> m: the 0x80 bias keeps borrows inside each byte, the
          // XOR removes it.  For G = 8 the common factor 2 of G - 2n is dropped (s (4 - n): all
          // scores halved alike, same order) so that the weights still fit a signed byte.
          const uint32_t sc = 16u >> m;
          const uint32_t gb = GMAX == 8 ? (uint32_t)G / 2u : (uint32_t)G, nm = GMAX == 8 ? 1u : 2u;
          out[w][m] = (int)((((sc * gb) * 0x01010101u | 0x80808080u) - nm * sc * n) ^ 0x80808080u);
        }
    };
    // the weights of every column set from the block's codes qx (lane = token): column set cs
    // needs the codes of step 32 cs + col, which the lane itself or its partner lane ^ 32 holds
    auto make_all_weights = [&](const uint32_t (&qx)[GMAX][W], v4i_t (&out)[NCS][W]) __attribute__((always_inline)) {
      if constexpr (NCS == 1) {
        make_weights(qx, out[0]);
      } else {
        uint32_t qo[GMAX][W];
#pragma unroll
        for (int g = 0; g < GMAX; ++g)
#pragma unroll
          for (int w = 0; w < W; ++w) qo[g][w] = (uint32_t)__shfl_xor((int)qx[g][w], 32);
#pragma unroll
        for (int cs = 0; cs < NCS; ++cs) {
          uint32_t qs[GMAX][W];
#pragma unroll
          for (int g = 0; g < GMAX; ++g)
#pragma unroll
            for (int w = 0; w < W; ++w) qs[g][w] = half == cs ? qx[g][w] : qo[g][w];
          make_weights(qs, out[cs]);
        }
      }
    };
    // The weights are the same in every wave (they depend on the lane and the block's query
    // codes only).  After the first block one wave that does not walk works them out for the
    // NEXT block while the walker walks (the codes were fetched a block ahead) and leaves them
    // in LDS; the barrier that ends the walk publishes them.
    v4i_t wt[NCS][W];
    if (wt_shared) {
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
        for (int w = 0; w < W; ++w)
#pragma unroll
          for (int m = 0; m < 4; ++m) wt[cs][w][m] = s_wt[((cs * W + w) * 4 + m) * 64 + lane];
    } else {
      make_all_weights(qc, wt);
    }

    // ---- every wave: its tiles against all T steps, running best per step ----------------
    // Slots are the rows of the product and steps its columns, so a lane holds, for ONE step
    // (its column), the scores of 16 slots of the tile (rows 8 (v / 4) + 4 half + v % 4).  One
    // more MFMA adds 15 - v to slot row v's score (scaled by 16 above), so the plain maximum
    // of the lane's 16 accumulators is already "largest score, then lowest slot", and a tile
    // costs eight 3-way maxima instead of a key and a comparison per value.  The same extra
    // MFMA pushes slots that may not win (past the end, sinks) far below every real score.
    // Running key per lane = (score, 2047 - tile, rank); the bias joins the tile term.
    const int rank = 15 - (4 * (col >> 3) + (col & 3));   // of slot row `col` in its lane
    v4i_t one_b;   // second operand of the extra MFMA: 1 at k = 0, 127 at k = 1..15 (half 0 only)
    one_b[0] = half == 0 ? 0x7F7F7F01 : 0;
    one_b[1] = one_b[2] = one_b[3] = half == 0 ? 0x7F7F7F7F : 0;
    int best[NCS], second[NCS];   // the lane's two largest group keys so far, per column set
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs) { best[cs] = 0; second[cs] = 0; }
    // the maximum of a tile's accumulators as a running key (score, lower tile, rank): the rank
    // moves below the tile number
    auto fold = [&](const v16i_t &acc, int tile, int &best, int &second) __attribute__((always_inline)) {
      int m0 = max(max(acc[0], acc[1]), acc[2]);
      int m1 = max(max(acc[3], acc[4]), acc[5]);
      int m2 = max(max(acc[6], acc[7]), acc[8]);
      int m3 = max(max(acc[9], acc[10]), acc[11]);
      int m4 = max(max(acc[12], acc[13]), acc[14]);
      m0 = max(max(m0, m1), m2);
      m3 = max(max(m3, m4), acc[15]);
      m0 = max(m0, m3);
      const uint32_t rk = (uint32_t)m0 & 15u;
      const uint32_t koff = ((uint32_t)(16 * bias) << 11) + ((uint32_t)((kMfmaMaxTiles - 1) - tile) << 4);
      const int key = (int)((((uint32_t)m0 & ~15u) << 11) + koff + rk);
      const int lo = best < key ? best : key;
      best = best > key ? best : key;
      second = second > lo ? second : lo;
    };
    // Tiles whose 32 slots all exist and may all win (no sink among them) take the short form:
    // no per-slot condition, the extra MFMA's first operand is the same for every tile, and
    // the next tile's code words are read from LDS before the current tile is multiplied.
    const int t_lo = MASKED ? (a.n_sink + 31) / 32 : 0, t_hi = C / 32;
    {
      v4i_t idx_f;
      idx_f[0] = half == 0 ? rank : 0;
      idx_f[1] = idx_f[2] = idx_f[3] = 0;
      int tile = wave + (t_lo - wave + WAVES - 1) / WAVES * WAVES;   // the wave's first tile >= t_lo
      if (tile < wave) tile = wave;
      uint32_t cw[W], nw[W];
      if (tile < t_hi) {
#pragma unroll
        for (int w = 0; w < W; ++w) cw[w] = tab[(size_t)(tile * 32 + col) * W + w];
      }
      for (; tile < t_hi; tile += WAVES) {
        const int nt = tile + WAVES < t_hi ? tile + WAVES : tile;
#pragma unroll
        for (int w = 0; w < W; ++w) nw[w] = tab[(size_t)(nt * 32 + col) * W + w];
        v4i_t cb[W];   // the slots' bits as operand bytes: once per tile, used by every column set
#pragma unroll
        for (int w = 0; w < W; ++w) cb[w] = spread16(cw[w], half);
#pragma unroll
        for (int cs = 0; cs < NCS; ++cs) {
          v16i_t acc = (v16i_t)(0);
#pragma unroll
          for (int w = 0; w < W; ++w)
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(cb[w], wt[cs][w], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(idx_f, one_b, acc, 0, 0, 0);
          fold(acc, tile, best[cs], second[cs]);
        }
#pragma unroll
        for (int w = 0; w < W; ++w) cw[w] = nw[w];
      }
    }
    // the other tiles (sinks at the front, a partial tile at the end): per-slot conditions
    for (int tile = wave; tile < n_tiles; tile += WAVES) {
      if (tile >= t_lo && tile < t_hi) {   // skip the full tiles in one stride-aligned jump
        const int skip = (t_hi - tile + WAVES - 1) / WAVES * WAVES;
        tile += skip - WAVES;
        continue;
      }
      const int slot = tile * 32 + col;
      const bool in = slot < C && (!MASKED || slot >= a.n_sink);   // sinks never leave slots 0 ..
      v4i_t cb[W];
#pragma unroll
      for (int w = 0; w < W; ++w) cb[w] = spread16(in ? tab[(size_t)slot * W + w] : 0u, half);
      // first operand of the extra MFMA: the rank at k = 0; -128 at k = 1..15 for a slot that
      // may not win (15 * -128 * 127 swamps any score)
      v4i_t idx_a;
      idx_a[0] = half == 0 ? (in ? rank : (int)0x80808000u) : 0;
      idx_a[1] = idx_a[2] = idx_a[3] = (half == 0 && !in) ? (int)0x80808080u : 0;
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs) {
        v16i_t acc = (v16i_t)(0);
#pragma unroll
        for (int w = 0; w < W; ++w)
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(cb[w], wt[cs][w], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(idx_a, one_b, acc, 0, 0, 0);
        fold(acc, tile, best[cs], second[cs]);
      }
    }
    // the lane's best as ((score + 1) << 20 | ~slot), the larger of the two halves, to LDS
    // a running key (score + bias) << 15 | (2047 - tile) << 4 | 15 - v as ((score + 1) << 20 | ~slot)
    auto final_key = [&](int rk) __attribute__((always_inline)) {
      const int v = 15 - (int)((uint32_t)rk & 15u);
      const uint32_t tile = (kMfmaMaxTiles - 1) - (((uint32_t)rk >> 4) & (kMfmaMaxTiles - 1));
      const uint32_t slot = tile * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
      return rk > 0 ? ((((uint32_t)rk >> 15) + 1u) << 20) | (0xFFFFFu - slot) : 0u;
    };
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs) {
      const uint32_t f1 = final_key(best[cs]), f2 = final_key(second[cs]);
      const uint32_t oth = (uint32_t)__shfl_xor((int)f1, 32);
      const int step = cs * 32 + col;
      if (half == 0) s_part[wave * T + step] = (int)(f1 > oth ? f1 : oth);
      s_cand[step * NCAND + (wave * 2 + half) * 2] = f1;
      s_cand[step * NCAND + (wave * 2 + half) * 2 + 1] = f2;
    }
    LSHE_STAT(const unsigned long long st_t2 = __builtin_amdgcn_s_memrealtime(); st_tiles += st_t2 - st_t0;)
    // the block's own tokens (rows) against the block's steps (columns)
    int own_best = -1;   // lane i (< T): best score for step i among the block's tokens old enough
    if (walker) {
      int ob[NCS];
      // token set ts (rows: tokens 32 ts + 8 (v / 4) + 4 half + v % 4) against step set cs >= ts
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs) ob[cs] = -1;
#pragma unroll
      for (int ts = 0; ts < NCS; ++ts) {
        v4i_t kb[W];   // key code of token 32 ts + col: the lane's own or its partner's
#pragma unroll
        for (int w = 0; w < W; ++w) {
          uint32_t kx = kc[w];
          if constexpr (NCS > 1) {
            const uint32_t ko = (uint32_t)__shfl_xor((int)kc[w], 32);
            kx = half == ts ? kc[w] : ko;
          }
          kb[w] = spread16(kx, half);
        }
#pragma unroll
        for (int cs = ts; cs < NCS; ++cs) {
          v16i_t acc = (v16i_t)(0);
#pragma unroll
          for (int w = 0; w < W; ++w)
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kb[w], wt[cs][w], acc, 0, 0, 0);
          // a token counts for a step if it came before it (and, with protected recent tokens,
          // at least n_recent steps before it)
          const int step = cs * 32 + col;
          const int last_h = step - (MASKED ? a.n_recent : 0) - 32 * ts - 4 * half;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int x = (acc[v] >> 4) + bias;   // acc = 16 x score
            s_new[step * SNS + 32 * ts + 8 * (v / 4) + 4 * half + v % 4] = (int16_t)x;
            ob[cs] = (8 * (v / 4) + v % 4 < last_h && x > ob[cs]) ? x : ob[cs];
          }
        }
      }
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs) {
        const int oth = __shfl_xor(ob[cs], 32);
        ob[cs] = ob[cs] > oth ? ob[cs] : oth;
      }
      own_best = ob[NCS == 1 ? 0 : half];   // lane = step: its column set is its half
    }
    __syncthreads();
    const bool share_next = WAVES > 1 && t0 + T < TE;
    if (share_next && wave == (turn + 1) % WAVES) {
      v4i_t wn[NCS][W];
      make_all_weights(qn, wn);
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
        for (int w = 0; w < W; ++w)
#pragma unroll
          for (int m = 0; m < 4; ++m) s_wt[((cs * W + w) * 4 + m) * 64 + lane] = wn[cs][w][m];
    }

    // ---- the steps of the block in order ------------------------------------------------------
    // The walker places runs of steps that simply take their block-start winner, and handles
    // alone the steps that cannot: an own token of the block may win, or the winner is gone (its
    // slot was written earlier in the block, or holds a protected recent token).  A step whose
    // winner is gone is decided from the candidate groups (head of this kernel); when that proof
    // fails, the step needs the whole table as it now stands, and every wave scores its share of
    // it (scan_table) before the walker goes on.  When queries repeat exactly, step after step
    // exhausts its candidates: after a block with kMfmaStaleLimit such steps the next
    // kMfmaDirectBlocks blocks are taken step by step (twice as many each time the block tried
    // after such a run is bad again).
    uint32_t ko_vec = 0;   // lane i: key ((score + 1) << 20 | ~slot) of step i's best old slot
    int ev = -1;           // lane j: the slot the block's token j went to (-1 not yet, -2 evicted again)
    int i = 0;             // the walker's next step
    int n_stale = 0;       // steps of this block the walker could not take on its own
    // Before the walk, for all steps at once (lane i = step i): the old winner's key, whether
    // it is a protected recent token (positions as at the start of the block; if the slot is
    // overwritten during the block the step is rescored anyway), and whether any of the block's
    // own earlier tokens could beat it on score alone.  The walk itself then runs on registers.
    uint64_t recent_mask = 0, own_mask = 0;
    bool special = true;   // lane i: step i cannot simply take its old winner (or is no step)
    LSHE_STAT(const unsigned long long st_t1 = __builtin_amdgcn_s_memrealtime(); st_bar += st_t1 - st_t2;)
    if (walker) {
      // From here to the end of the walk this wave is the unit's critical path (its other
      // waves wait at the barrier below): it goes ahead of other units' waves on its SIMD.
      __builtin_amdgcn_s_setprio(3);
      bool recent = false, own = false;
      if (lane < T) {
        for (int p = 0; p < WAVES; ++p) {
          const uint32_t o = (uint32_t)s_part[p * T + lane];
          ko_vec = ko_vec > o ? ko_vec : o;
        }
        if constexpr (MASKED)
          recent = ko_vec != 0u && pos[0xFFFFFu - (ko_vec & 0xFFFFFu)] > t0 + lane - 1 - a.n_recent;
        const int ms = own_best;
        own = ms >= 0 && ((((uint32_t)ms + 1u) << 20) | 0xFFFFFu) > ko_vec;
        special = lane >= n_steps || ko_vec == 0u || recent || own;
      }
      recent_mask = __builtin_amdgcn_ballot_w64(recent);
      own_mask = __builtin_amdgcn_ballot_w64(own);
      LSHE_STAT(st_pa += __builtin_amdgcn_s_memrealtime() - st_t1;)
    }
    const int so_vec = (int)(0xFFFFFu - (ko_vec & 0xFFFFFu));   // lane i: step i's old winner's slot
    const int so_word = ko_vec != 0u ? so_vec >> 5 : 0;   // (lanes without a winner read word 0)
    // Steps of the block that share an old winner: the later one finds it written when its turn
    // comes.  All but one of the steps with the same winner are made special -- which one is
    // left out does not matter: a special step ends the run of steps placed together, so two
    // steps with one winner are never placed in the same run, and whether a step's winner is
    // gone is read from the bit map of written slots when the step is reached.  Found with one
    // LDS atomic per lane: of the lanes that set the same bit, all but one see it set.
    uint64_t dup_mask = 0;
    if (walker) {
      bool dup = false;
      if (lane < T && ko_vec != 0u) {
        const uint32_t bit = 1u << (so_vec & 31);
        dup = (atomicOr(&s_seen[so_word], bit) & bit) != 0u;
        atomicAnd(&s_seen[so_word], ~bit);
      }
      special = special || dup;
      dup_mask = __builtin_amdgcn_ballot_w64(dup);
    }
    auto take = [&](int e, int step) __attribute__((always_inline)) {   // walker only
      ev = ev == e ? -2 : ev;
      if (lane == step) ev = e;
      store_token(e, step);
    };
    for (;;) {
      if (walker) {
        __builtin_amdgcn_s_setprio(3);
        LSHE_STAT(st_t0 = __builtin_amdgcn_s_memrealtime(); if (i == 0) st_pre += st_t0 - st_t1;)
        while (i < n_steps) {
          LSHE_STAT(++st_pass;)
          // Most steps just take their old winner, and such steps do not interact: step i's
          // winner stands if it is not the slot an earlier step of the block wrote to.  Flag,
          // for all steps at once, the ones that are special or whose winner was written by a
          // token already placed (the bit map of written slots); steps whose winner an earlier
          // unplaced step shares are special already.  The steps before the first flagged one
          // are then placed together.
          const bool gone = ((s_written[so_word] >> (so_vec & 31)) & 1u) != 0u;
          uint64_t gone_mask = __builtin_amdgcn_ballot_w64(gone);
          uint64_t fm = __builtin_amdgcn_ballot_w64(special || gone || lane >= T);
          fm &= ~0ull << i;
          const int s = fm != 0 ? (int)__builtin_ctzll(fm) : T;   // lanes >= n_steps are flagged: s <= n_steps
          if (lane >= i && lane < s) {
            const int e = so_vec;
            ev = e;
#pragma unroll
            for (int w = 0; w < W; ++w) tab[(size_t)e * W + w] = kc[w];
            if constexpr (MASKED) pos[e] = t0 + lane;
            spos[e] = t0 + lane;
            if (a.evict_log) a.evict_log[(size_t)u * NQ + (t0 + lane - C)] = e;
            atomicOr(&s_written[e >> 5], 1u << (e & 31));
          }
          i = s;
          if (i >= n_steps) break;
          // step i on its own
          const uint32_t ko = (uint32_t)__builtin_amdgcn_readlane((int)ko_vec, i);
          LSHE_STAT(++st_single;)
          if (ko == 0u) break;   // no old slot may be evicted: the table as it stands, all waves
          if ((dup_mask >> i) & 1) {
            // a step of this very run may have taken the winner: look again
            const int so_i = (int)(0xFFFFFu - (ko & 0xFFFFFu));
            if ((s_written[so_i >> 5] >> (so_i & 31)) & 1u) gone_mask |= 1ull << i;
          }
          // the block's own earlier tokens that still sit in a slot (and are old enough)
          const int sn = lane < T ? (int)s_new[i * SNS + lane] : 0;
          const uint32_t kn2 = (lane + (MASKED ? a.n_recent : 0) < i && ev >= 0)
                                   ? ((((uint32_t)sn + 1u) << 20) | (0xFFFFFu - (uint32_t)ev)) : 0u;
          uint32_t win = ko;
          if (((recent_mask | gone_mask) >> i) & 1) {
            // The old winner is gone (or protected): the step's candidate groups, see the head of
            // this kernel.  Lane c < NCAND takes candidate c; odd c are the second maxima.
            LSHE_STAT(++st_conf;)
            const int newest_evictable = t0 + i - 1 - a.n_recent;
            const int so_i = (int)(0xFFFFFu - (ko & 0xFFFFFu));
            // everything that does not depend on another load goes out together: the candidates'
            // keys, and -- since the old winner's own group is certainly among the groups to score
            // again -- that group's 16 slots (lanes 0 .. 15: rows 8 (v / 4) + 4 half + v % 4)
            const uint32_t fin = lane < NCAND ? s_cand[i * NCAND + lane] : 0u;
            const int s0 = (so_i & ~31) + 8 * ((lane >> 2) & 3) + (so_i & 4) + (lane & 3);
            bool ok0 = lane < 16 && s0 < C && (!MASKED || s0 >= a.n_sink);
            uint32_t cw0[W] = {};
            if (ok0) {
              ok0 = ((s_written[s0 >> 5] >> (s0 & 31)) & 1u) == 0u;
              if constexpr (MASKED) ok0 = ok0 && pos[s0] <= newest_evictable;
#pragma unroll
              for (int w = 0; w < W; ++w) cw0[w] = tab[(size_t)s0 * W + w];
            }
            // the step's query codes and their popcount: the block's scores are
            // sum_b c_b (G - 2 n_b) + bias = Hamming distance - sum_b n_b + bias (halved for G = 8)
            uint32_t qi[GMAX][W];
            int nq = 0;
#pragma unroll
            for (int g = 0; g < GMAX; ++g)
#pragma unroll
              for (int w = 0; w < W; ++w) {
                qi[g][w] = (uint32_t)__builtin_amdgcn_readlane((int)qc[g][w], i);
                nq += __popc(qi[g][w]);   // (codes of heads >= G are zero)
              }
            auto group_key = [&](bool okx, int sx, const uint32_t (&cwx)[W]) __attribute__((always_inline)) {
              int ham = 0;
#pragma unroll
              for (int w = 0; w < W; ++w)
#pragma unroll
                for (int g = 0; g < GMAX; ++g)
                  if (g < G) ham += __popc(cwx[w] ^ qi[g][w]);
              const int sb = (GMAX == 8 ? (ham - nq) >> 1 : ham - nq) + bias;
              return okx ? (((uint32_t)sb + 1u) << 20) | (0xFFFFFu - (uint32_t)sx) : 0u;
            };
            // the candidates: listed slots that still stand
            const bool has = fin != 0u;
            const int cslot = (int)(0xFFFFFu - (fin & 0xFFFFFu));
            bool ok = false;
            if (has) {
              ok = ((s_written[cslot >> 5] >> (cslot & 31)) & 1u) == 0u;
              if constexpr (MASKED) ok = ok && pos[cslot] <= newest_evictable;
            }
            uint32_t x = ok ? fin : kn2;
            x = x > kn2 ? x : kn2;
            const uint32_t k0 = group_key(ok0, s0, cw0);
            x = x > k0 ? x : k0;
            // other listed groups whose best slot is gone: scored again one by one (rare)
            uint64_t redo = __builtin_amdgcn_ballot_w64(has && !ok && ((cslot ^ so_i) & ~0x1B) != 0);
            while (redo != 0) {
              const int c = (int)__builtin_ctzll(redo);
              redo &= redo - 1;
              const int rs = __builtin_amdgcn_readlane(cslot, c);
              const int s2 = (rs & ~31) + 8 * ((lane >> 2) & 3) + (rs & 4) + (lane & 3);
              bool ok2 = lane < 16 && s2 < C && (!MASKED || s2 >= a.n_sink);
              uint32_t cw2[W] = {};
              if (ok2) {
                ok2 = ((s_written[s2 >> 5] >> (s2 & 31)) & 1u) == 0u;
                if constexpr (MASKED) ok2 = ok2 && pos[s2] <= newest_evictable;
#pragma unroll
                for (int w = 0; w < W; ++w) cw2[w] = tab[(size_t)s2 * W + w];
              }
              const uint32_t k2 = group_key(ok2, s2, cw2);
              x = x > k2 ? x : k2;
            }
            win = wave_max_u32(x);
            // proof: no partition's second maximum (odd lanes) lies above the candidate found
            if (win == 0u || __builtin_amdgcn_ballot_w64((lane & 1) && fin > win) != 0)
              break;   // not decided by the candidates: all waves
          } else if ((own_mask >> i) & 1) {
            if (__builtin_amdgcn_ballot_w64(kn2 > ko) != 0) win = wave_max_u32(kn2);
          }
          take(key_slot(win), i);
          ++i;
        }
        if (lane == 0) {
          s_flag[0] = (uint32_t)i;
          s_flag[1 + WAVES] = n_stale >= kMfmaStaleLimit ? (uint32_t)kMfmaDirectBlocks : 0u;
        }
        // block done: the written-slot bits go back to zero (a token evicted again has ev = -2;
        // its slot's bit belongs to the token that took the slot after it)
        if (i >= n_steps && lane < T && ev >= 0) atomicAnd(&s_written[ev >> 5], ~(1u << (ev & 31)));
        LSHE_STAT(st_walk += __builtin_amdgcn_s_memrealtime() - st_t0;)
        __builtin_amdgcn_s_setprio(0);
      }
      __syncthreads();   // also: the walker's table writes are visible to everyone
      const int ri = (int)s_flag[0];
      if (ri >= n_steps) {
        // (every wave keeps the same count: a unit whose queries stay correlated soon stops
        // paying for trial blocks)
        if (s_flag[1 + WAVES] != 0u) {
          direct_left = direct_run;
          direct_run = direct_run < 1024 ? 2 * direct_run : direct_run;
        } else {
          direct_run = kMfmaDirectBlocks;
        }
        LSHE_STAT(st_block += __builtin_amdgcn_s_memrealtime() - st_tb;)
        wt_shared = share_next;
        break;
      }
      // step ri on the table as it stands: its plane masks from its query codes, then all waves
      uint32_t qi[GMAX][W];
#pragma unroll
      for (int g = 0; g < GMAX; ++g)
#pragma unroll
        for (int w = 0; w < W; ++w) qi[g][w] = (uint32_t)__builtin_amdgcn_readlane((int)qc[g][w], ri);
      Planes<W, NP> pl;
      make_planes<W, NP, GMAX>(qi, G, P0, pl);
      const uint32_t win = scan_table(pl, t0 + ri);
      if (walker) {
        if (win != 0u) take(key_slot(win), ri);
        i = ri + 1;
        ++n_stale;
        LSHE_STAT(++st_fall;)
      }
      __syncthreads();   // the slot's new code is in place before anyone scores again
    }
  }
  if (TE < N) {   // more launches follow: leave the table where the next one finds it
    for (int s = tid; s < C * W; s += NT) saved[s] = tab[s];
  }
  if (tid == 0) a.n_valid[u] = C;
#ifdef LSHE_STAMPS
  if (lane == 0 && u < kStampGroups && wave < kStampWaves) {
    unsigned long long *o = g_stamps[u][wave];
    o[0] = st_tiles; o[1] = st_walk; o[2] = st_block; o[3] = st_pass; o[4] = st_single; o[5] = st_conf;
    o[6] = st_fall; o[7] = st_bar; o[8] = st_pre; o[9] = st_pa;
  }
#endif
}

// ---- L2-norm policy: the sequential stage as a two-level tournament per unit -------------------
// The comparator's score does not depend on the query, so a step need not look at every slot.
// One wave per unit.  LDS holds tab[slot] = norm bits + 1 for the slots that may be evicted now,
// 0 for the others (first n_sink tokens, recent tokens), and a ring of the n_recent + 1 newest
// tokens {slot, norm bits + 1}.  The slots are cut into 64 contiguous groups of GS = 2^k; lane g
// keeps the best (norm, lowest slot) of group g in registers, the unit's best is a register-only
// wave reduction over those, cached while no group changes.  At step t the token t - 1 - n_recent
// leaves the ring and becomes evictable; if it beats the cached best it is the victim itself and
// nothing else changes (about half of the steps on the benchmark shapes); otherwise the best
// slot goes, the aged token's norm enters tab and its group's maximum, and only the victim's
// group is read again (GS words, one LDS round trip) before the unit's best is reduced anew.
// Token t takes the victim's slot and enters the ring.  Victims equal the slot-by-slot
// definition, ties included ((norm, ~slot) keys are unique).
struct L2Best {
  uint32_t hi, lo;   // norm bits + 1 (0 = nothing evictable), 0xFFFFFFFF - slot
};
__device__ __forceinline__ bool l2_better(uint32_t hi, uint32_t lo, const L2Best &b) {
  return hi > b.hi || (hi == b.hi && lo > b.lo);
}
// the lanes' candidates -> the wave's best, in every lane (two 32-bit maxima for the 64-bit key)
__device__ __forceinline__ L2Best l2_wave_best(const L2Best &mine) {
  L2Best w;
  w.hi = wave_max_u32(mine.hi);
  w.lo = wave_max_u32(mine.hi == w.hi ? mine.lo : 0u);
  return w;
}

__global__ __launch_bounds__(64) void evict_l2_kernel(const EvictArgs a, int log2gs) {
  extern __shared__ __align__(16) uint32_t l2_lds[];
  const int lane = threadIdx.x;
  const int C = a.C, N = a.N, NQ = N - C, R = a.n_recent, S = a.n_sink;
  const int GS = 1 << log2gs;                       // 64 * GS >= C
  uint32_t *tab = l2_lds;                           // [64 * GS]
  uint2 *ring = (uint2 *)(tab + 64 * GS);           // [R + 1] {slot, norm bits + 1}
  const long long u = blockIdx.x;
  const uint32_t *ck = a.codes_k + (size_t)u * N;
  int32_t *spos = a.slot_pos + (size_t)u * C;

  // ---- the first C tokens fill the slots in order ---------------------------------------------
  for (int s = lane; s < 64 * GS; s += 64) {
    uint32_t v = 0;
    if (s < C) {
      spos[s] = s;
      const uint32_t key = ck[s] + 1u;
      if (s > C - 2 - R) ring[s % (R + 1)] = make_uint2((uint32_t)s, key);   // (these are >= n_sink)
      else if (s >= S) v = key;
    }
    tab[s] = v;
  }
  __syncthreads();

  // best of group g by all lanes; ascending slots per lane, so a strict comparison keeps the lowest
  auto rescan = [&](int g) __attribute__((always_inline)) {
    L2Best b = {0u, 0u};
    for (int j = lane; j < GS; j += 64) {
      const uint32_t v = tab[g * GS + j];
      if (v > b.hi) { b.hi = v; b.lo = 0xFFFFFFFFu - (uint32_t)(g * GS + j); }
    }
    return l2_wave_best(b);
  };
  L2Best mine = {0u, 0u};   // lane g: best of group g
  for (int g = 0; g < 64; ++g) {
    const L2Best b = rescan(g);
    if (lane == g) mine = b;
  }
  L2Best top = l2_wave_best(mine);

  // ---- tokens C .. N-1; their norms are fetched 64 at a time, one chunk ahead -------------------
  uint32_t kn = C + lane < N ? ck[C + lane] : 0u;
  int ri = C % (R + 1);   // ring index of token t (and of the token t - 1 - R it replaces)
  for (int tb = C; tb < N; tb += 64) {
    const uint32_t kc = kn;
    if (tb + 64 < N) kn = tb + 64 + lane < N ? ck[tb + 64 + lane] : 0u;
    const int tend = tb + 64 < N ? tb + 64 : N;
    for (int t = tb; t < tend; ++t) {
      const uint32_t nk = (uint32_t)__builtin_amdgcn_readlane((int)kc, t - tb) + 1u;
      const uint2 aged = ring[ri];   // token t - 1 - R becomes evictable now (same word in every lane)
      const uint32_t aslot = (uint32_t)__builtin_amdgcn_readfirstlane((int)aged.x);
      const uint32_t akey = (uint32_t)__builtin_amdgcn_readfirstlane((int)aged.y);
      uint32_t e = aslot;
      if (!l2_better(akey, 0xFFFFFFFFu - aslot, top)) {   // uniform: the cached best goes
        e = 0xFFFFFFFFu - top.lo;
        if (lane == 0) { tab[aslot] = akey; tab[e] = 0u; }
        const int ga = (int)(aslot >> log2gs), ge = (int)(e >> log2gs);
        if (lane == ga && l2_better(akey, 0xFFFFFFFFu - aslot, mine)) { mine.hi = akey; mine.lo = 0xFFFFFFFFu - aslot; }
        const L2Best b = rescan(ge);   // reads tab after lane 0's writes: one wave, LDS in order
        if (lane == ge) mine = b;
        top = l2_wave_best(mine);
      }
      if (lane == 0) {
        ring[ri] = make_uint2(e, nk);   // token t takes the victim's slot
        spos[e] = t;
        if (a.evict_log) a.evict_log[(size_t)u * NQ + (t - C)] = (int32_t)e;
      }
      ri = ri + 1 == R + 1 ? 0 : ri + 1;
    }
  }
  if (lane == 0) a.n_valid[u] = C;
}

// ---- any budget: code table in global memory (the output code cache itself) ------------------
__global__ __launch_bounds__(1024) void evict_global_kernel(const EvictArgs a, int W) {
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int C = a.C, N = a.N, G = a.G, NQ = N - C;
  const uint32_t *ck = a.codes_k + (size_t)u * N * W;
  const uint32_t *cq = a.codes_q + (size_t)u * G * NQ * W;
  uint32_t *tab = a.code_cache + (size_t)u * C * W;
  int32_t *spos = a.slot_pos + (size_t)u * C;
  __shared__ uint32_t s_best[2][16];
  for (int s = tid; s < C; s += 1024) {
    for (int w = 0; w < W; ++w) tab[(size_t)s * W + w] = ck[(size_t)s * W + w];
    spos[s] = s;
  }
  __syncthreads();
  for (int t = C; t < N; ++t) {
    uint32_t best = 0;
    const int newest_evictable = t - 1 - a.n_recent;
    for (int s = tid; s < C; s += 1024) {
      uint32_t sc = 0;
      for (int w = 0; w < W; ++w) {
        const uint32_t c = tab[(size_t)s * W + w];
        for (int g = 0; g < G; ++g) sc += __popc(c ^ cq[((size_t)g * NQ + (t - C)) * W + w]);
      }
      const int p = spos[s];
      const bool ok = p >= a.n_sink && p <= newest_evictable;
      const uint32_t key = ok ? make_key(sc, (uint32_t)s) : 0u;
      best = best > key ? best : key;
    }
    best = wave_max_u32(best);
    if (lane == 0) s_best[t & 1][wave] = best;
    __syncthreads();   // also orders this step's table reads before the write below
    for (int k = 0; k < 16; ++k) {
      const uint32_t o = s_best[t & 1][k];
      best = best > o ? best : o;
    }
    if (best != 0u && tid == 0) {
      const int e = key_slot(best);
      for (int w = 0; w < W; ++w) tab[(size_t)e * W + w] = ck[(size_t)t * W + w];
      spos[e] = t;
      if (a.evict_log) a.evict_log[(size_t)u * NQ + (t - C)] = e;
    }
    __syncthreads();   // the write is visible to the whole workgroup before the next step reads
  }
  if (tid == 0) a.n_valid[u] = C;
}

// ---- prompts that fit the budget: tokens go to slots in order ---------------------------------
__global__ void fill_positions_kernel(int32_t *slot_pos, int32_t *n_valid, long long units, int C,
                                      int N) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < units * C) {
    const int s = (int)(i % C);
    slot_pos[i] = s < N ? s : -1;
  }
  if (i < units) n_valid[i] = N < C ? N : C;
}

// ---- gather survivors: K_cache[s] <- K_prompt[slot_pos[s]], same for V and the codes ---------
// TPR threads move one row (16 bytes each); empty slots are zero-filled.
template <int TPR>
__global__ __launch_bounds__(256) void gather_kernel(const uint4 *__restrict__ Kp,
                                                     const uint4 *__restrict__ Vp,
                                                     const uint32_t *__restrict__ codes_k,
                                                     const int32_t *__restrict__ slot_pos,
                                                     uint4 *__restrict__ Kc, uint4 *__restrict__ Vc,
                                                     uint32_t *__restrict__ code_cache,
                                                     long long n_slots, int C, int N, int W,
                                                     int write_codes) {
  const long long gs = ((long long)blockIdx.x * 256 + threadIdx.x) / TPR;   // global slot
  const int part = threadIdx.x % TPR;
  if (gs >= n_slots) return;
  const long long u = gs / C;
  const int src = slot_pos[gs];
  uint4 k = make_uint4(0, 0, 0, 0), v = make_uint4(0, 0, 0, 0);
  if (src >= 0) {
    k = Kp[((size_t)u * N + src) * TPR + part];
    v = Vp[((size_t)u * N + src) * TPR + part];
  }
  Kc[(size_t)gs * TPR + part] = k;
  Vc[(size_t)gs * TPR + part] = v;
  if (write_codes && part < W)
    code_cache[(size_t)gs * W + part] = src >= 0 ? codes_k[((size_t)u * N + src) * W + part] : 0u;
}

// LDS bytes of evict_lds_kernel for a config
static size_t evict_lds_bytes(const Dims &m, bool masked, int waves) {
  size_t words = (size_t)m.C * m.W + (masked ? (size_t)m.C : 0);
  words += words & 1;
  return (words + 2 * (size_t)waves) * 4;
}

constexpr size_t kLdsPerGroupMax = 160 * 1024 - 512;   // LDS of one CU, minus slack

template <int W, int NP, int WAVES>
static int launch_evict_lds(const Dims &m, const EvictArgs &a, hipStream_t st) {
  const bool masked = (m.n_sink | m.n_recent) != 0;
  const int P0 = m.G == 1 ? 0 : 1;
  const size_t lds = evict_lds_bytes(m, masked, WAVES);
  const dim3 grid((unsigned)m.units), block(64 * WAVES);
  if (masked) {
    auto k = evict_lds_kernel<W, NP, true, WAVES>;
    if (lds > 48 * 1024)
      LSHE_HIP_TRY(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(k, grid, block, lds, st, a, P0);
  } else {
    auto k = evict_lds_kernel<W, NP, false, WAVES>;
    if (lds > 48 * 1024)
      LSHE_HIP_TRY(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(k, grid, block, lds, st, a, P0);
  }
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

template <int W, int WAVES>
static int launch_evict_np(const Dims &m, const EvictArgs &a, hipStream_t st) {
  if (m.G <= 2) return launch_evict_lds<W, 1, WAVES>(m, a, st);
  if (m.G == 4) return launch_evict_lds<W, 2, WAVES>(m, a, st);
  return launch_evict_lds<W, 3, WAVES>(m, a, st);
}

// Waves per unit.  A step is bound by the integer ALUs plus a serial tail (reduction, slot
// update), so it pays to split a unit's table over more waves until the chip holds about
// eight waves per SIMD (8192) -- as long as every lane keeps at least eight slots, below
// which the per-step tail and the barrier dominate (measured on 2048 and 256 units).
static int evict_waves(const Dims &m) {
  int waves = 1;
  while (waves < 16 && m.units * waves * 2 <= 8192 && (int64_t)waves * 2 * 64 * 8 <= m.C) waves *= 2;
  return waves;
}

// The matrix-core kernel: budgets worth a block of 32 steps per pass, and hashes wide enough
// that scores do not tie all the time: with very few bits many slots share the top score, the
// lowest of them wins step after step, and most steps of a block find their block-start winner
// overwritten.  The candidate lists absorb much of that (measured, prompt compression of 256
// units x 2048 slots / eviction phase of 2048 units x 2458 slots against the vector-ALU
// kernel: 8 bits 1.19 / 5.4 ms against 1.39 / 10.8 ms, 12 bits 0.74 / 3.2 against 1.40 / 10.5);
// at 4 bits the small workload is still slower (1.84 against 1.40 ms), so the floor is 8.
constexpr int kMfmaMinBudget = 512;
constexpr int kMfmaMinBits = 8;
constexpr int kMfmaMaxGroup = 8;   // the weights must fit a signed byte: 16 (G - 2n) up to G = 4, 16 (4 - n) for G = 8
static size_t evict_mfma_lds_bytes(const Dims &m, int waves) {
  const size_t T = kMfmaSteps;
  const bool masked = (m.n_sink | m.n_recent) != 0;
  return ((size_t)m.C * m.W + (size_t)waves * T + T * (T + 2) / 2 + 2 + (size_t)waves +
          T * 4 * (size_t)waves + 2 * ((size_t)(m.C + 31) / 32) + (T / 32) * 4 * (size_t)m.W * 64 +
          (masked ? (size_t)m.C : 0)) * 4;
}
template <int W, int WAVES, int GMAX>
static int launch_evict_mfma_g(const Dims &m, const EvictArgs &a, hipStream_t st) {
  const size_t lds = evict_mfma_lds_bytes(m, WAVES);
  const int P0 = m.G == 1 ? 0 : 1;
  const dim3 grid((unsigned)m.units), block(64 * WAVES);
  if ((m.n_sink | m.n_recent) != 0) {
    auto k = evict_mfma_kernel<W, WAVES, GMAX, true>;
    if (lds > 48 * 1024)
      LSHE_HIP_TRY(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(k, grid, block, lds, st, a, P0);
  } else {
    auto k = evict_mfma_kernel<W, WAVES, GMAX, false>;
    if (lds > 48 * 1024)
      LSHE_HIP_TRY(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(k, grid, block, lds, st, a, P0);
  }
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}
template <int W, int WAVES>
static int launch_evict_mfma(const Dims &m, const EvictArgs &a, hipStream_t st) {
  if (m.G <= 2) return launch_evict_mfma_g<W, WAVES, 2>(m, a, st);
  if (m.G <= 4) return launch_evict_mfma_g<W, WAVES, 4>(m, a, st);
  return launch_evict_mfma_g<W, WAVES, 8>(m, a, st);
}

static bool evict_uses_mfma(const Dims &m) {
  return m.G <= kMfmaMaxGroup && m.r >= kMfmaMinBits && m.C >= kMfmaMinBudget &&
         m.C <= 32 * kMfmaMaxTiles && evict_mfma_lds_bytes(m, evict_waves(m)) <= kLdsPerGroupMax;
}
// HashEvict's sequential stage keeps the code table in LDS when it fits, else works on the
// output code cache in global memory (which the gather then leaves alone)
static bool evict_table_in_lds(const Dims &m) {
  const bool masked = (m.n_sink | m.n_recent) != 0;
  return evict_uses_mfma(m) || evict_lds_bytes(m, masked, evict_waves(m)) <= kLdsPerGroupMax;
}

// returns LSHE_UNSUPPORTED when the table does not fit LDS (the caller then uses the
// global-memory kernel)
template <int W>
static int launch_evict(const Dims &m, const EvictArgs &a, hipStream_t st) {
  const bool masked = (m.n_sink | m.n_recent) != 0;
  const int waves = evict_waves(m);
  if (evict_uses_mfma(m)) {
    switch (waves) {
      case 1: return launch_evict_mfma<W, 1>(m, a, st);
      case 2: return launch_evict_mfma<W, 2>(m, a, st);
      case 4: return launch_evict_mfma<W, 4>(m, a, st);
      case 8: return launch_evict_mfma<W, 8>(m, a, st);
      default: return launch_evict_mfma<W, 16>(m, a, st);
    }
  }
  if (evict_lds_bytes(m, masked, waves) > kLdsPerGroupMax) return LSHE_UNSUPPORTED;
  switch (waves) {
    case 1: return launch_evict_np<W, 1>(m, a, st);
    case 2: return launch_evict_np<W, 2>(m, a, st);
    case 4: return launch_evict_np<W, 4>(m, a, st);
    case 8: return launch_evict_np<W, 8>(m, a, st);
    default: return launch_evict_np<W, 16>(m, a, st);
  }
}

// evict_l2_kernel: slots per group (a power of two, 64 groups cover the budget) and LDS bytes
static int evict_l2_log2gs(const Dims &m) {
  int k = 0;
  while ((64 << k) < m.C) ++k;
  return k;
}
static size_t evict_l2_lds_bytes(const Dims &m) {
  return ((size_t)64 << evict_l2_log2gs(m)) * 4 + ((size_t)m.n_recent + 1) * 8;
}

static int launch_evict_l2(const Dims &m, const EvictArgs &a, hipStream_t st) {
  const size_t lds = evict_l2_lds_bytes(m);
  if (lds > kLdsPerGroupMax) return LSHE_UNSUPPORTED;
  if (lds > 48 * 1024)
    LSHE_HIP_TRY(hipFuncSetAttribute((const void *)evict_l2_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(evict_l2_kernel, dim3((unsigned)m.units), dim3(64), lds, st, a, evict_l2_log2gs(m));
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

// ---- long prompts: the query hashing beside the eviction ------------------------------------------
// Hashing the queries is bound by HBM, the eviction by vector-ALU issue, and the eviction of
// token t needs only the query codes up to t.  A whole call on many units therefore cuts the
// tokens >= C into ranges: a second stream of the library's hashes the queries range by range
// while the caller's stream hashes the keys and then evicts range by range, each launch waiting
// only for its own range's codes (evict_mfma_kernel carries its table from launch to launch in
// code_cache and slot_pos; the gather overwrites code_cache at the end anyway).  Same results:
// the kernel is exact whatever its blocks are.  Not under stream capture, and only for the
// matrix-core eviction kernel.
constexpr int kRangesAuto = 8;          // ranges of a long prompt
constexpr int kRangesMax = 16;
constexpr int kRangeMinSteps = 4096;    // shorter prompts, or fewer units, stay in one piece: measured,
constexpr int kRangeMinUnits = 512;     // 256 units x 2048 steps lose 12 %, 1024 x 2048 and 256 x 5734 gain nothing
constexpr int kSideStreamDevices = 64;
static std::atomic<int> g_prefill_ranges{0};   // test hook: 0 = automatic
static hipStream_t g_side_stream[kSideStreamDevices];
static std::mutex g_side_mutex;

static int side_stream(hipStream_t *out) {
  int dev = -1;
  LSHE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kSideStreamDevices) return LSHE_HIP_ERROR;
  std::lock_guard<std::mutex> lock(g_side_mutex);
  if (!g_side_stream[dev]) LSHE_HIP_TRY(hipStreamCreateWithFlags(&g_side_stream[dev], hipStreamNonBlocking));
  *out = g_side_stream[dev];
  return LSHE_OK;
}

static int prefill_ranges(const Dims &m, int N, hipStream_t st) {
  const int NQ = N - m.C;
  const int forced = g_prefill_ranges.load(std::memory_order_relaxed);
  int n = forced > 0 ? forced : (NQ >= kRangeMinSteps && m.units >= kRangeMinUnits ? kRangesAuto : 1);
  if (n > kRangesMax) n = kRangesMax;
  if (n > NQ / kMfmaSteps) n = NQ / kMfmaSteps;   // at least one block of steps per range
  if (n < 2) return 1;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return 1;
  return n;
}

struct RangeEvents {   // events of one call, released when the call returns (HIP frees them once they have fired)
  hipEvent_t ev[kRangesMax + 1];
  int n = 0;
  int create(int count) {
    for (; n < count; ++n) LSHE_HIP_TRY(hipEventCreateWithFlags(&ev[n], hipEventDisableTiming));
    return LSHE_OK;
  }
  ~RangeEvents() {
    for (int i = 0; i < n; ++i) (void)hipEventDestroy(ev[i]);
  }
};

// The three stages of the prompt stage; lshe_prefill_compress runs all of them.
static int prefill_common(const lshe_config *cfg, const void *R_dev, const void *K_prompt,
                          const void *V_prompt, const void *Q_prompt, int32_t n_prompt,
                          void *K_cache, void *V_cache, uint32_t *code_cache, int32_t *slot_pos,
                          int32_t *n_valid, int32_t *evict_log, void *workspace,
                          size_t workspace_bytes, void *stream, int phases) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (n_prompt < 0) return LSHE_INVALID_ARG;
  if ((phases & ~(LSHE_PREFILL_HASH | LSHE_PREFILL_EVICT | LSHE_PREFILL_GATHER)) != 0 || phases == 0)
    return LSHE_INVALID_ARG;
  if (!K_cache || !V_cache || !code_cache || !slot_pos || !n_valid) return LSHE_INVALID_ARG;
  if (!R_dev && cfg->policy != LSHE_POLICY_L2NORM) return LSHE_INVALID_ARG;
  const Dims m = dims_of(cfg);
  if (m.G != 1 && m.G != 2 && m.G != 4 && m.G != 8) return LSHE_UNSUPPORTED;
  const int N = n_prompt, C = m.C;
  if (N > 0 && (!K_prompt || !V_prompt)) return LSHE_INVALID_ARG;
  const bool l2 = m.policy == LSHE_POLICY_L2NORM;
  if (N > C && !Q_prompt && !l2) return LSHE_INVALID_ARG;
  // the comparator's sequential stage has no kernel for tables beyond one CU's LDS: say so
  // before anything is enqueued
  if (l2 && N > C && evict_l2_lds_bytes(m) > kLdsPerGroupMax) return LSHE_UNSUPPORTED;
  if (N > 0) {
    if (!workspace) return LSHE_INVALID_ARG;
    if (workspace_bytes < prefill_ws_bytes(m, N)) return LSHE_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255u) != 0) return LSHE_INVALID_ARG;
  }
  const int tpr = m.d * m.esize / 16;
  if (tpr != 8 && tpr != 16 && tpr != 32) return LSHE_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  const long long n_slots = (long long)m.units * C;

  uint32_t *codes_k = N > 0 ? (uint32_t *)((char *)workspace + kWsHeaderBytes) : nullptr;
  uint32_t *codes_q =
      N > 0 ? (uint32_t *)((char *)codes_k + align_up((size_t)m.units * N * m.W * 4, 256)) : nullptr;

  const bool whole = phases == (LSHE_PREFILL_HASH | LSHE_PREFILL_EVICT | LSHE_PREFILL_GATHER);
  const int n_ranges = (whole && N > C && !l2 && evict_uses_mfma(m)) ? prefill_ranges(m, N, st) : 1;
  if (n_ranges > 1) {
    hipStream_t side = nullptr;
    rc = side_stream(&side);
    if (rc != LSHE_OK) return rc;
    RangeEvents e;
    rc = e.create(n_ranges + 1);
    if (rc != LSHE_OK) return rc;
    const int NQ = N - C;
    const int len = ((NQ + n_ranges - 1) / n_ranges + kMfmaSteps - 1) / kMfmaSteps * kMfmaSteps;
    // the side stream starts where the caller's stream stands
    LSHE_HIP_TRY(hipEventRecord(e.ev[n_ranges], st));
    LSHE_HIP_TRY(hipStreamWaitEvent(side, e.ev[n_ranges], 0));
    for (int j = 0; j < n_ranges; ++j) {
      const int b = C + j * len, t1 = b + len < N ? b + len : N;
      if (b >= N) { LSHE_HIP_TRY(hipEventRecord(e.ev[j], side)); continue; }
      if (j == 1) {   // the keys beyond the first range, before the second range's event
        const int kb = C + len;
        rc = hash_rows(m, R_dev, K_prompt, m.units * (int64_t)(N - kb), N - kb, N, kb, codes_k, side, N, kb);
        if (rc != LSHE_OK) return rc;
      }
      rc = hash_rows(m, R_dev, Q_prompt, m.units * m.G * (int64_t)(t1 - b), t1 - b, N, b, codes_q, side, NQ,
                     b - C);
      if (rc != LSHE_OK) return rc;
      LSHE_HIP_TRY(hipEventRecord(e.ev[j], side));
    }
    // the keys of the slots' first tokens and of the first range on the caller's stream, so that the
    // first eviction starts early; the rest in one launch on the side stream
    {
      const int k1 = C + len < N ? C + len : N;
      rc = hash_rows(m, R_dev, K_prompt, m.units * (int64_t)k1, k1, N, 0, codes_k, st, N, 0);
      if (rc != LSHE_OK) return rc;
    }
    EvictArgs a;
    a.codes_k = codes_k; a.codes_q = codes_q; a.code_cache = code_cache;
    a.slot_pos = slot_pos; a.n_valid = n_valid; a.evict_log = evict_log;
    a.C = C; a.G = m.G; a.N = N; a.n_sink = m.n_sink; a.n_recent = m.n_recent;
    a.units = m.units;
    for (int j = 0; j < n_ranges; ++j) {
      const int b = C + j * len, t1 = b + len < N ? b + len : N;
      LSHE_HIP_TRY(hipStreamWaitEvent(st, e.ev[j], 0));   // (every one of them: the side stream is joined)
      if (b >= N) continue;
      a.t_begin = b; a.t_end = t1;
      rc = m.W == 1 ? launch_evict<1>(m, a, st) : launch_evict<2>(m, a, st);
      if (rc != LSHE_OK) return rc;
    }
    phases = LSHE_PREFILL_GATHER;
  }
  // ---- eq. (2) for every prompt key and for the queries of tokens >= C ----------------------
  if ((phases & LSHE_PREFILL_HASH) && N > 0) {
    rc = l2 ? norm_rows(m, K_prompt, m.units * N, codes_k, st)
            : hash_rows(m, R_dev, K_prompt, m.units * N, m.units * N, m.units * N, 0, codes_k, st);
    if (rc != LSHE_OK) return rc;
    if (N > C && !l2) {
      rc = hash_rows(m, R_dev, Q_prompt, m.units * m.G * (int64_t)(N - C), N - C, N, C, codes_q, st);
      if (rc != LSHE_OK) return rc;
    }
  }
  // ---- Algorithm 1 steps 1-5 token by token, on the codes alone ------------------------------
  const bool table_in_lds = l2 || evict_table_in_lds(m);
  if (phases & LSHE_PREFILL_EVICT) {
    if (N > C) {
      EvictArgs a;
      a.codes_k = codes_k; a.codes_q = l2 ? nullptr : codes_q; a.code_cache = code_cache;
      a.slot_pos = slot_pos; a.n_valid = n_valid; a.evict_log = evict_log;
      a.C = C; a.G = m.G; a.N = N; a.n_sink = m.n_sink; a.n_recent = m.n_recent;
      a.units = m.units;
      a.t_begin = C; a.t_end = N;
      if (l2) {
        rc = launch_evict_l2(m, a, st);
      } else if (table_in_lds) {
        rc = m.W == 1 ? launch_evict<1>(m, a, st) : launch_evict<2>(m, a, st);
      } else {
        hipLaunchKernelGGL(evict_global_kernel, dim3((unsigned)m.units), dim3(1024), 0, st, a, m.W);
        rc = hipGetLastError() == hipSuccess ? LSHE_OK : LSHE_HIP_ERROR;
      }
      if (rc != LSHE_OK) return rc;
    } else {
      const long long n = n_slots > m.units ? n_slots : m.units;
      hipLaunchKernelGGL(fill_positions_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                         slot_pos, n_valid, (long long)m.units, C, N);
      LSHE_HIP_TRY(hipGetLastError());
    }
  }
  // ---- survivors' keys, values and codes into the slot arrays -----------------------------------
  if (phases & LSHE_PREFILL_GATHER) {
    const bool codes_written = N > C && !table_in_lds;   // the global-memory kernel worked in place
    const long long threads = n_slots * tpr;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
#define LSHE_GATHER(TPR_)                                                                        \
  hipLaunchKernelGGL((gather_kernel<TPR_>), grid, block, 0, st, (const uint4 *)K_prompt,         \
                     (const uint4 *)V_prompt, codes_k, slot_pos, (uint4 *)K_cache,               \
                     (uint4 *)V_cache, code_cache, n_slots, C, N, m.W, codes_written ? 0 : 1)
    switch (tpr) {
      case 8: LSHE_GATHER(8); break;
      case 16: LSHE_GATHER(16); break;
      default: LSHE_GATHER(32); break;
    }
#undef LSHE_GATHER
    LSHE_HIP_TRY(hipGetLastError());
  }
  return LSHE_OK;
}

}  // namespace lshe

using namespace lshe;

extern "C" const char *lshe_prefill_plan(const lshe_config *cfg, int32_t n_prompt) {
  if (lshe_check_config(cfg) != LSHE_OK || n_prompt < 0) return nullptr;
  const Dims m = dims_of(cfg);
  const bool l2 = m.policy == LSHE_POLICY_L2NORM;
  if (n_prompt == 0) return "fill_positions_kernel + gather_kernel";
  if (n_prompt <= m.C)
    return l2 ? "norm_rows_kernel + fill_positions_kernel + gather_kernel"
              : "hash_rows_kernel + fill_positions_kernel + gather_kernel";
  if (l2)
    return evict_l2_lds_bytes(m) > kLdsPerGroupMax ? nullptr
                                                  : "norm_rows_kernel + evict_l2_kernel + gather_kernel";
  if (evict_uses_mfma(m)) return "hash_rows_kernel x2 + evict_mfma_kernel + gather_kernel";
  if (evict_table_in_lds(m)) return "hash_rows_kernel x2 + evict_lds_kernel + gather_kernel";
  return "hash_rows_kernel x2 + evict_global_kernel + gather_kernel";
}

extern "C" void lshe_debug_prefill_ranges(int32_t n) {
  g_prefill_ranges.store(n > 0 ? n : 0, std::memory_order_relaxed);
}

extern "C" int lshe_prefill_compress(const lshe_config *cfg, const void *R_dev,
                                     const void *K_prompt, const void *V_prompt,
                                     const void *Q_prompt, int32_t n_prompt, void *K_cache,
                                     void *V_cache, uint32_t *code_cache, int32_t *slot_pos,
                                     int32_t *n_valid, int32_t *evict_log, void *workspace,
                                     size_t workspace_bytes, void *stream) {
  return prefill_common(cfg, R_dev, K_prompt, V_prompt, Q_prompt, n_prompt, K_cache, V_cache,
                        code_cache, slot_pos, n_valid, evict_log, workspace, workspace_bytes, stream,
                        LSHE_PREFILL_HASH | LSHE_PREFILL_EVICT | LSHE_PREFILL_GATHER);
}

extern "C" int lshe_prefill_phases(const lshe_config *cfg, const void *R_dev,
                                   const void *K_prompt, const void *V_prompt,
                                   const void *Q_prompt, int32_t n_prompt, void *K_cache,
                                   void *V_cache, uint32_t *code_cache, int32_t *slot_pos,
                                   int32_t *n_valid, int32_t *evict_log, void *workspace,
                                   size_t workspace_bytes, void *stream, int32_t phases) {
  return prefill_common(cfg, R_dev, K_prompt, V_prompt, Q_prompt, n_prompt, K_cache, V_cache,
                        code_cache, slot_pos, n_valid, evict_log, workspace, workspace_bytes, stream,
                        phases);
}

#ifdef LSHE_STAMPS
// instrumented build only: the prompt-stage kernels' counters, copied to the host
extern "C" int lshe_read_stamps_prefill(unsigned long long *host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(lshe::g_stamps), bytes);
}
#endif
