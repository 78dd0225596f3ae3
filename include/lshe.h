/*
 * lshe -- HashEvict's pre-attention KV-cache eviction path on AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only; every DEVICE buffer is owned by the
 * caller (allocate it with any HIP allocator); the library allocates no memory,
 * host or device, keeps no state between calls, never synchronises the host
 * with the device and enqueues all work on the HIP stream passed as `stream` (a
 * hipStream_t cast to void*; NULL = the default stream).  The one HOST pointer
 * in the interface (R_host of lshe_init_projection) is read before that call
 * returns.
 *
 * Notation (Section 3 of the paper unless noted):
 *   d  head dimension            r  hash bits (the paper's c / b), W = ceil(r/32)
 *   C  cache budget in slots     G  query heads per KV head (GQA group)
 *   H  KV heads per layer        L  layers covered by one call       B  sequences
 * A *unit* is one (sequence, layer, KV head); units are independent and are laid
 * out contiguously in [B][L][H] order in every buffer.  Per unit the cache is C
 * fixed slots: keys K[C][d], values V[C][d], hash codes code[C][W] (uint32, bit j
 * of a code at bit j%32 of word j/32, unused high bits 0), slot_pos[C] (index of
 * the token a slot holds, -1 = empty) and n_valid (occupied slots; slots
 * 0..n_valid-1 are the occupied ones).
 *
 * Return value of every function: LSHE_OK or a negative lshe_status.  On an
 * argument error nothing is enqueued and no buffer is touched.
 */
#ifndef LSHE_H
#define LSHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lshe_status {
  LSHE_OK = 0,
  LSHE_INVALID_ARG = -1,          /* NULL required pointer, value out of range */
  LSHE_UNSUPPORTED = -2,          /* a shape this build has no kernel for */
  LSHE_WORKSPACE_TOO_SMALL = -3,
  LSHE_HIP_ERROR = -4,            /* a HIP runtime call (launch, copy) failed */
  LSHE_SCRATCH_EXCEEDED = -5      /* lshe_decode_step_noalloc: the configuration needs more scratch
                                     memory than the library's built-in array holds */
} lshe_status;

enum { LSHE_F32 = 0, LSHE_BF16 = 1 };

/* Which score decides the victim.
 *   LSHE_POLICY_HASH    HashEvict (Section 3): summed Hamming distance between the cached key
 *                       codes and the current query codes; the largest distance is evicted.
 *   LSHE_POLICY_L2NORM  the attention-free comparator the paper measures against (Sections 1,
 *                       2.1, 4): the key with the largest L2 norm is evicted.  A slot's code is
 *                       then ONE word, the bit pattern of the key's squared norm summed in fp32
 *                       (see lshe_key_norms; W = 1 whatever hash_bits says; R_dev and the
 *                       queries play no part in the selection).  fp32 summation is within
 *                       d * 2^-24 relative of the exact norm, so between two keys whose norms
 *                       are closer than that the choice is not defined by the paper's rule and
 *                       may differ from an evaluation in higher precision.  Everything else --
 *                       slots, ties to the lowest slot, kept first / recent tokens, attention --
 *                       is the same.  Budgets above 32,768 slots (whose table of norms, padded
 *                       to 64 groups of a power of two, does not fit one CU's LDS) are
 *                       LSHE_UNSUPPORTED in lshe_prefill_compress under this policy. */
enum { LSHE_POLICY_HASH = 0, LSHE_POLICY_L2NORM = 1 };

/* Plain data, passed by const pointer and read during the call only. */
typedef struct lshe_config {
  int32_t head_dim;    /* d: 64 or 128 */
  int32_t hash_bits;   /* r in [1, 64] */
  int32_t n_kv_heads;  /* H >= 1 */
  int32_t gqa_group;   /* G: 1, 2, 4 or 8 (others in [1, 16] are LSHE_UNSUPPORTED); Hamming scores are
                          summed over the group */
  int32_t n_layers;    /* L >= 1 */
  int32_t batch;       /* B >= 1 */
  int32_t budget;      /* C in [1, 2^20); C > n_sink + n_recent */
  int32_t dtype;       /* LSHE_F32 or LSHE_BF16: element type of K, V, Q, out and of R_dev */
  int32_t n_sink;      /* first tokens that are never evicted (Section 4 set-up uses 4); >= 0 */
  int32_t n_recent;    /* most recent tokens that are never evicted (Section 4: 10); >= 0 */
  int32_t policy;      /* LSHE_POLICY_HASH or LSHE_POLICY_L2NORM */
} lshe_config;

/* Helpers (host only, no device work). */
const char *lshe_strerror(int status);
const char *lshe_version(void);
/* 0 if cfg is valid, else the status the entry points would return. */
int lshe_check_config(const lshe_config *cfg);
/* Bytes of R_dev: 32*W rows of d elements of cfg->dtype.  0 on invalid cfg. */
size_t lshe_projection_bytes(const lshe_config *cfg);
/* Bytes of the per-unit code cache summed over all units: B*L*H*C*W*4
 * (Section 3, Complexity: C*b bits per head, rounded up to whole words). */
size_t lshe_code_cache_bytes(const lshe_config *cfg);
/* Names of the kernels one lshe_decode_step call launches for this configuration (the plan
 * depends on the number of units, the budget, the group size, the hash width and the element
 * type, never on the data; a profile lists these names).  NULL on an invalid or unsupported
 * cfg.  The string is static.  Present plans: "decode_fused_solo_kernel", "decode_fused_kernel"
 * (one launch), "attn_local_kernel + merge_small_kernel", "attn_local_kernel + merge_local_kernel"
 * (at most / more than 32 slot ranges per unit) and "select_kernel + attn_kernel" (two launches). */
const char *lshe_decode_plan(const lshe_config *cfg);
/* The same for one lshe_prefill_compress call with prompts of n_prompt tokens ("hash_rows_kernel
 * x2" = one launch for the keys, one for the queries; a long prompt on many units runs the same
 * kernels in token ranges, see lshe_prefill_compress).  NULL on an invalid or unsupported cfg. */
const char *lshe_prefill_plan(const lshe_config *cfg, int32_t n_prompt);
/* Workspace needed by lshe_decode_step (n_prompt = 0) or by both
 * lshe_decode_step and lshe_prefill_compress with prompts of n_prompt tokens.
 * The first int32 of a workspace is its STATUS WORD (the rest of the first 256 bytes is unused,
 * every other use of the workspace starts behind them).  Kernels only ever OR bits into it, and
 * only when something went wrong inside a kernel; nothing in the library reads or clears it.  A
 * caller who wants to watch it sets it to 0 once after allocating the workspace and reads it
 * whenever it synchronises with the stream anyway:
 *   LSHE_STATUS_SELECT_TIMEOUT  a bounded wait inside the single-kernel decode step expired (the
 *       waves that stream K/V poll for the slot that the selecting wave publishes; the poll count
 *       is limited so that an internal error ends in a wrong `out` and this bit, never in a
 *       kernel that does not finish).  Not reachable in a correct build. */
enum { LSHE_STATUS_SELECT_TIMEOUT = 1 };
size_t lshe_workspace_bytes(const lshe_config *cfg, int32_t n_prompt);
/* For the library's own tests of that give-up path, process-wide: spin_limit > 0 = number of polls
 * before a streaming wave gives up (0 restores the default, several seconds' worth);
 * withhold_victim != 0 makes the selecting wave NOT publish the slot, so that every streaming
 * wave runs into the limit, sets the status bit and leaves through the normal exit (the step's
 * `out` is then wrong by design; caches, `evicted` and every other output are still right).
 * Never call this in production code. */
void lshe_debug_select_wait(int32_t spin_limit, int32_t withhold_victim);
/* For the library's own tests, process-wide: lshe_prefill_compress cuts the tokens beyond the
 * budget into n ranges whenever its matrix-core eviction kernel runs (0 restores the automatic
 * choice: 8 ranges for prompts at least 4096 tokens longer than the budget on at least 512
 * units, else one; see lshe_prefill_compress).  The results do not depend on it. */
void lshe_debug_prefill_ranges(int32_t n);

/*
 * Random projection matrix R of Section 2 (i.i.d. N(0,1), r hyperplanes in R^d),
 * fixed for the lifetime of a cache because stored key codes are compared with
 * later query codes.
 *   R_host  HOST, nullable: [d][r] row-major float (column j = hyperplane j); read
 *           before the call returns (it may be freed or changed right after).  If NULL
 *           the matrix is generated on the host from `seed` by a counter-based
 *           generator: element (i, j) is the Box-Muller cosine branch of two
 *           uniforms taken from splitmix64(seed, 2*(i*r+j)) and (..., +1).
 *   R_dev   DEVICE, out: lshe_projection_bytes(cfg) bytes.  Layout [32*W][d], row j =
 *           hyperplane j in cfg->dtype (rounded to nearest-even for bf16), rows >= r
 *           zero.  This is the only form the other entry points read; a test that
 *           needs the values the device uses reads this buffer back.
 * Like every other entry point the call allocates nothing and does not wait for the
 * device: the values travel to the device as arguments of a few small kernels enqueued
 * on `stream` (one per 960 elements), which store them transposed and rounded.
 */
int lshe_init_projection(const lshe_config *cfg, uint64_t seed, const float *R_host,
                         void *R_dev, void *stream);

/*
 * Section 2, eq. (2): codes[t] = pack(sgn(R x_t)), sgn(z) = 1 if z >= 0 else 0.
 *   X      DEVICE [n][d] in cfg->dtype, rows contiguous
 *   codes  DEVICE out [n][W] uint32
 * Products are accumulated in fp32 on the matrix cores (bf16 inputs are exact
 * products); a bit whose projection is within rounding of zero may differ from an
 * exact evaluation.  n = 0 is a no-op.  Only head_dim, hash_bits, dtype of cfg are used
 * (the eviction policy plays no part: the result is always eq. (2)).
 */
int lshe_hash_keys(const lshe_config *cfg, const void *R_dev, const void *X, int64_t n,
                   uint32_t *codes, void *stream);

/*
 * The score of the L2-norm comparator (Sections 1, 2.1 and the baselines of Section 4: keys
 * with a large L2 norm are evicted first): norm2[t] = sum_i x_t[i]^2, the squared norm, which
 * orders like the norm.
 *   X      DEVICE [n][d] in cfg->dtype, rows contiguous
 *   norm2  DEVICE out [n] float
 * Summed in fp32: eight elements per lane (bf16 products are exact), then a tree over the
 * d/8 lanes of a row -- within d * 2^-24 relative of the exact value.  These are the words
 * the code cache holds under LSHE_POLICY_L2NORM (viewed as uint32: non-negative floats order
 * like their bit patterns).  n = 0 is a no-op.  Only head_dim and dtype of cfg are used.
 */
int lshe_key_norms(const lshe_config *cfg, const void *X, int64_t n, float *norm2, void *stream);

/*
 * Prompt Encoding Stage (Section 3): per unit, the first min(N, C) prompt tokens fill
 * slots in order; each later token t runs steps 1-5 of Algorithm 1 with its own
 * queries (victim = evictable slot with the largest summed Hamming distance to the G
 * query codes of token t, lowest slot on ties; the token's key, value and code
 * overwrite that slot).  Attention outputs of prompt tokens are not produced.
 *   K_prompt, V_prompt  DEVICE [B][L][H][N][d]
 *   Q_prompt            DEVICE [B][L][H*G][N][d]; query head h*G+g belongs to KV head h;
 *                       only tokens >= C are read; may be NULL when N <= C
 *   K_cache, V_cache    DEVICE out [B][L][H][C][d]
 *   code_cache          DEVICE out [B][L][H][C][W]
 *   slot_pos            DEVICE out [B][L][H][C]   (-1 for empty slots)
 *   n_valid             DEVICE out [B][L][H]      (= min(N, C))
 *   evict_log           DEVICE out, nullable [B][L][H][max(N-C,0)]: victim slot per token
 *   workspace           DEVICE, >= lshe_workspace_bytes(cfg, N) bytes, 256-byte aligned
 * Empty slots of K/V/code caches are zero-filled.  N = 0 gives empty caches.
 * Everything is enqueued on `stream` in order, with one exception that a caller does not see:
 * for prompts at least 4096 tokens longer than the budget on at least 512 units (and not under
 * stream capture) the query hashing runs on a second stream that the library creates once per
 * device (default priority, non-blocking), forked from `stream` at the call and joined to it
 * before the call's last kernels, so that it overlaps the eviction; work enqueued on `stream`
 * after the call is ordered behind all of it as usual.
 */
int lshe_prefill_compress(const lshe_config *cfg, const void *R_dev,
                          const void *K_prompt, const void *V_prompt, const void *Q_prompt,
                          int32_t n_prompt,
                          void *K_cache, void *V_cache, uint32_t *code_cache,
                          int32_t *slot_pos, int32_t *n_valid, int32_t *evict_log,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * The three stages of lshe_prefill_compress as separate calls, for callers that want to put
 * other work (or timing events) between them.  `phases` is a sum of
 *   LSHE_PREFILL_HASH    eq. (2) for every prompt key and for the queries of tokens >= C, into
 *                        the workspace (LSHE_POLICY_L2NORM: the keys' squared norms);
 *   LSHE_PREFILL_EVICT   Algorithm 1 steps 1-5 token by token on those codes alone: writes
 *                        slot_pos, n_valid and evict_log;
 *   LSHE_PREFILL_GATHER  the surviving tokens' keys, values and codes into K_cache, V_cache and
 *                        code_cache.
 * The stages of one prompt, called in this order on one stream with the same arguments and the
 * same workspace (whose contents carry the codes from stage to stage), leave exactly what
 * lshe_prefill_compress leaves; all arguments have the meaning given there and are checked
 * alike for every stage.  phases = 0 or other bits: LSHE_INVALID_ARG.
 */
enum { LSHE_PREFILL_HASH = 1, LSHE_PREFILL_EVICT = 2, LSHE_PREFILL_GATHER = 4 };
int lshe_prefill_phases(const lshe_config *cfg, const void *R_dev,
                        const void *K_prompt, const void *V_prompt, const void *Q_prompt,
                        int32_t n_prompt,
                        void *K_cache, void *V_cache, uint32_t *code_cache,
                        int32_t *slot_pos, int32_t *n_valid, int32_t *evict_log,
                        void *workspace, size_t workspace_bytes, void *stream, int32_t phases);

/*
 * One time step of Algorithm 1 ("Decoding Stage") for every unit:
 *   1. hash the G current queries and the new key (eq. 2);
 *   2. score[s] = sum over g of d_H(code[s], h(q_g)) for occupied slots (eq. 5, negated);
 *   3. e = n_valid if the cache is not full (append), else the evictable slot with the
 *      largest score, lowest slot on ties (eq. 6); a slot is evictable unless it holds
 *      one of the first n_sink tokens or one of the n_recent tokens before t;
 *   4. K[e], V[e], code[e], slot_pos[e] <- k_new, v_new, h(k_new), t; n_valid grows to at most C;
 *   5. out[g] = softmax(q_g K^T / sqrt(d)) V over the occupied slots of the updated
 *      cache (eq. 1), fp32 accumulation, stored in cfg->dtype.
 *   q_new        DEVICE [B][L][H*G][d]
 *   k_new,v_new  DEVICE [B][L][H][d]
 *   pos          DEVICE [B] int32: token index t of this step for each sequence
 *   K_cache .. n_valid   DEVICE in/out, layouts as in lshe_prefill_compress
 *   out          DEVICE out [B][L][H*G][d]
 *   evicted      DEVICE out, nullable [B][L][H]: slot written this step
 *   scores_dbg   DEVICE out, nullable [B][L][H][C] int32: step-2 scores (-1 for slots that
 *                were empty before the step)
 *   codes_dbg    DEVICE out, nullable [B][L][H][G+1][W]: the G query codes then the key code
 *   evicted_mass DEVICE out, nullable [B][L][H*G] float: the attention-loss diagnostic of
 *                Section 4.8 per step -- the softmax probability (eq. 1 scaling) that query head
 *                g puts on the evicted token among the C keys cached before the step plus the
 *                new key; 0 while the cache is still filling
 *   workspace    DEVICE, >= lshe_workspace_bytes(cfg, 0) bytes, 256-byte aligned; contents
 *                need not be preserved or initialised between calls (its first int32 is the
 *                status word described at lshe_workspace_bytes)
 * Calls on the same cache must be ordered (same stream, or otherwise serialised).
 * The call only launches kernels (no memset, copy, allocation or synchronisation) and reads the
 * token position from device memory, so it may be captured in a HIP graph and replayed for
 * later steps with the inputs updated in place.
 * K_cache and V_cache must be 16-byte aligned.  code_cache and slot_pos need 4-byte alignment
 * only, but the fastest plan (see lshe_decode_plan) reads them as 16-byte vectors and is
 * skipped when they are not 16-byte aligned.
 * The attention sum of a unit is split over the waves of a workgroup in an order that can
 * depend on timing, so the last bits of `out` (and of evicted_mass) may differ between two
 * runs on the same inputs; every other output is integer work and is reproducible.
 */
int lshe_decode_step(const lshe_config *cfg, const void *R_dev,
                     const void *q_new, const void *k_new, const void *v_new,
                     const int32_t *pos,
                     void *K_cache, void *V_cache, uint32_t *code_cache,
                     int32_t *slot_pos, int32_t *n_valid,
                     void *out, int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                     float *evicted_mass,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two halves of lshe_decode_step as separate calls, for callers that want to put other
 * work (or timing events) between them.  lshe_decode_select(...) followed by
 * lshe_decode_attend(...) on the same stream leaves the caches and `out` exactly as
 * lshe_decode_step(...) does (which, for configurations with many units, runs both halves in
 * a single kernel instead); arguments have the meaning given there.
 *   lshe_decode_select  steps 1-4 of the list above (Algorithm 1 steps 1-5): hash, score,
 *                       pick the victim, overwrite it in place.  Does not touch the workspace.
 *   lshe_decode_attend  step 5 (eq. 1, Algorithm 1 step 6): attention of the G queries of each
 *                       unit over its occupied slots; reads the caches only, so it may also be
 *                       called on its own.
 */
int lshe_decode_select(const lshe_config *cfg, const void *R_dev,
                       const void *q_new, const void *k_new, const void *v_new,
                       const int32_t *pos,
                       void *K_cache, void *V_cache, uint32_t *code_cache,
                       int32_t *slot_pos, int32_t *n_valid,
                       int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                       void *workspace, size_t workspace_bytes, void *stream);
int lshe_decode_attend(const lshe_config *cfg, const void *q_new,
                       const void *K_cache, const void *V_cache, const int32_t *n_valid,
                       void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * lshe_decode_select over a code table stored the way the paper's implementation stores it --
 * ONE BYTE PER HASH BIT (Sections 4.6 and 4.7; the paper names packing as future work) -- so
 * that what the packed table saves can be measured on the same hardware with the same select.
 *   code_bytes  DEVICE in/out [B][L][H][C][32*W] uint8: byte j of a slot is bit j of its code
 *               (0 or 1; bytes >= r are 0), 16-byte aligned
 *   slot_pos, n_valid, evicted, q_new, k_new, pos   as in lshe_decode_select
 * Steps 1-4 of lshe_decode_step for the code table and the positions only (the key / value
 * caches are not touched): the victim equals lshe_decode_select's on a packed table with the
 * same contents.  LSHE_POLICY_HASH, head_dim 128 and LSHE_BF16 only (LSHE_UNSUPPORTED otherwise).
 */
int lshe_decode_select_unpacked(const lshe_config *cfg, const void *R_dev,
                                const void *q_new, const void *k_new, const int32_t *pos,
                                uint8_t *code_bytes, int32_t *slot_pos, int32_t *n_valid,
                                int32_t *evicted, void *stream);

/*
 * lshe_decode_step for callers that cannot allocate device memory at all -- code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: the same step with
 * the same kernels, but the scratch memory that lshe_decode_step takes through `workspace`
 * (partial softmax states of the split plans, the victim's logits, the select's hand-over to
 * the merge kernel) lives in an array of LSHE_BUILTIN_SCRATCH_BYTES bytes inside the library's
 * device image.  Inputs, caches and outputs are still the caller's; all other arguments and
 * results are those of lshe_decode_step.
 *   - The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library
 *     routine) and does not synchronise.  The first call on a device looks the array's address
 *     up (hipGetSymbolAddress, with that device current) and keeps it for the process; make
 *     that first call outside a graph capture.
 *   - A configuration whose plan needs more than LSHE_BUILTIN_SCRATCH_BYTES of scratch returns
 *     LSHE_SCRATCH_EXCEEDED and does nothing (the need is lshe_workspace_bytes(cfg, 0) for the
 *     plans of several launches, 0 for the single-kernel plans, see lshe_decode_plan).  2 MiB
 *     covers every split-plan configuration with up to 4 query heads per KV head, and groups of
 *     8 query heads up to about 500 units.
 *   - Every call on a GPU uses that GPU's one array (each GPU the library runs on holds its own
 *     copy until the process ends): two calls that may overlap on one GPU -- different streams
 *     with no ordering between them -- race on it and give wrong outputs.  Calls on one stream,
 *     or otherwise ordered, are fine; nothing in the array has to be cleared between calls, for
 *     every word a step reads from it is written earlier in the same step.
 */
#define LSHE_BUILTIN_SCRATCH_BYTES ((size_t)2 << 20)
int lshe_decode_step_noalloc(const lshe_config *cfg, const void *R_dev,
                             const void *q_new, const void *k_new, const void *v_new,
                             const int32_t *pos,
                             void *K_cache, void *V_cache, uint32_t *code_cache,
                             int32_t *slot_pos, int32_t *n_valid,
                             void *out, int32_t *evicted, int32_t *scores_dbg, uint32_t *codes_dbg,
                             float *evicted_mass, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LSHE_H */
