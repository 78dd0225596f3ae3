// lshe_init_projection and lshe_hash_keys: the random projection matrix of Section 2 and
// the bulk sign-random-projection hashing kernel (eq. (2)) on the matrix cores.
#include <math.h>
#include <string.h>

#include "lshe_hash_tile.h"
#include "lshe_kernels.h"

namespace lshe {

// ---- host-side N(0,1) generator (documented in lshe.h) -----------------------------------
static inline uint64_t splitmix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

static inline double normal_at(uint64_t key, uint64_t idx) {
  const uint64_t a = splitmix64(key + 2 * idx);
  const uint64_t b = splitmix64(key + 2 * idx + 1);
  const double u1 = ((double)(a >> 11) + 1.0) * (1.0 / 9007199254740992.0);  // (0, 1]
  const double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);          // [0, 1)
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

// ---- bulk hashing kernel -------------------------------------------------------------------
// Rows are addressed as (segment s, index i): element offset (s*seg_stride + seg_off + i)*HD;
// the code of flattened row f = s*seg_len + i goes to output row s*out_stride + out_off + i
// (= f when a call covers whole segments).  One wavefront hashes 32 rows per iteration and
// strides over tiles, keeping its slice of R in registers (bf16).
template <int HD, int W, bool BF16>
__global__ __launch_bounds__(256) void hash_rows_kernel(const void *__restrict__ X,
                                                        const void *__restrict__ R_dev, int r,
                                                        long long n_rows, long long seg_len,
                                                        long long seg_stride, long long seg_off,
                                                        long long out_stride, long long out_off,
                                                        uint32_t *__restrict__ codes) {
  const int lane = threadIdx.x & 63;
  const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const long long n_waves = (long long)gridDim.x * (blockDim.x >> 6);
  const long long n_tiles = (n_rows + 31) / 32;
  constexpr int ES = BF16 ? 2 : 4;

  RFrag<HD, W, BF16> rf;
  rf.load(R_dev, lane);

  // address of this lane's row of a tile; rows past the end re-read the last row
  auto row_ptr = [&](long long tile) {
    long long f = tile * 32 + (lane & 31);
    f = f < n_rows ? f : n_rows - 1;
    const long long s = f / seg_len;
    const long long i = f - s * seg_len;
    return (const char *)X + (size_t)(s * seg_stride + seg_off + i) * HD * ES;
  };
  const bool whole_segments = out_stride == seg_len && out_off == 0;   // output row = flattened row

  // two tiles in flight: the next tile's rows are requested before the current tile is multiplied
  XFrag<HD, BF16> x[2];
  if (wave < n_tiles) x[0].load(row_ptr(wave), lane);
  for (long long tile = wave; tile < n_tiles; tile += 2 * n_waves) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const long long cur = tile + b * n_waves;
      if (cur >= n_tiles) break;
      const long long nxt = cur + n_waves;
      x[b ^ 1].load(row_ptr(nxt < n_tiles ? nxt : cur), lane);
      uint32_t code[W];
      hash_tile32<HD, W, BF16>(x[b], rf, r, lane, code);
      const long long f = cur * 32 + (lane & 31);
      if (lane < 32 && f < n_rows) {
        long long out_row = f;
        if (!whole_segments) {   // (uniform; only the calls that hash a token range of every segment)
          const long long s = f / seg_len;
          out_row = s * out_stride + out_off + (f - s * seg_len);
        }
#pragma unroll
        for (int w = 0; w < W; ++w) codes[(size_t)out_row * W + w] = code[w];
      }
    }
  }
}

template <int HD, int W, bool BF16>
static int launch_hash(const void *X, const void *R_dev, int r, int64_t n_rows, int64_t seg_len,
                       int64_t seg_stride, int64_t seg_off, int64_t out_stride, int64_t out_off,
                       uint32_t *codes, hipStream_t st) {
  const int64_t n_tiles = (n_rows + 31) / 32;
  int64_t blocks = (n_tiles + 3) / 4;
  const int64_t cap = 256 * 8;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL((hash_rows_kernel<HD, W, BF16>), dim3((unsigned)blocks), dim3(256), 0, st, X,
                     R_dev, r, (long long)n_rows, (long long)seg_len, (long long)seg_stride,
                     (long long)seg_off, (long long)out_stride, (long long)out_off, codes);
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

// ---- L2-norm comparator: the "code" of a row is the bit pattern of its squared norm ---------
// HD/8 lanes share a row (16 or 32 bytes each, so a wave-wide load reads 64/(HD/8) whole rows,
// contiguous memory); a wave keeps kNormRowsInFlight such loads in flight.  Bound: HBM read
// (HD*e bytes per row, 4 written).
constexpr int kNormRowsInFlight = 4;

template <int HD, bool BF16>
__global__ __launch_bounds__(256) void norm_rows_kernel(const void *__restrict__ X, long long n_rows,
                                                        uint32_t *__restrict__ codes) {
  constexpr int ES = BF16 ? 2 : 4;
  constexpr int LPR = HD / 8, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, c = lane % LPR, rg = lane / LPR;
  const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long row0 = wave * (RPW * kNormRowsInFlight) + rg;
  Raw8<BF16> x[kNormRowsInFlight];
#pragma unroll
  for (int k = 0; k < kNormRowsInFlight; ++k) {
    long long f = row0 + k * RPW;
    f = f < n_rows ? f : n_rows - 1;   // rows past the end re-read the last row
    x[k].load((const char *)X + ((size_t)f * HD + c * 8) * ES);
  }
#pragma unroll
  for (int k = 0; k < kNormRowsInFlight; ++k) {
    const uint32_t nb = norm2_bits_of_piece<HD, BF16>(x[k]);
    const long long f = row0 + k * RPW;
    if (c == 0 && f < n_rows) codes[f] = nb;
  }
}

int norm_rows(const Dims &m, const void *X, int64_t n_rows, uint32_t *codes, hipStream_t st) {
  if (n_rows <= 0) return LSHE_OK;
  const int rows_per_wave = 64 / (m.d / 8) * kNormRowsInFlight;
  const int64_t waves = (n_rows + rows_per_wave - 1) / rows_per_wave;
  const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  const bool bf = m.dtype == LSHE_BF16;
  if (m.d == 128) {
    if (bf) hipLaunchKernelGGL((norm_rows_kernel<128, true>), grid, block, 0, st, X, (long long)n_rows, codes);
    else hipLaunchKernelGGL((norm_rows_kernel<128, false>), grid, block, 0, st, X, (long long)n_rows, codes);
  } else if (m.d == 64) {
    if (bf) hipLaunchKernelGGL((norm_rows_kernel<64, true>), grid, block, 0, st, X, (long long)n_rows, codes);
    else hipLaunchKernelGGL((norm_rows_kernel<64, false>), grid, block, 0, st, X, (long long)n_rows, codes);
  } else {
    return LSHE_UNSUPPORTED;
  }
  LSHE_HIP_TRY(hipGetLastError());
  return LSHE_OK;
}

int hash_rows(const Dims &m, const void *R_dev, const void *X, int64_t n_rows, int64_t seg_len,
              int64_t seg_stride, int64_t seg_off, uint32_t *codes, hipStream_t st, int64_t out_stride,
              int64_t out_off) {
  if (out_stride < 0) { out_stride = seg_len; out_off = 0; }   // whole segments: output row = flattened row
  if (n_rows <= 0) return LSHE_OK;
  const bool bf = m.dtype == LSHE_BF16;
#define LSHE_HASH_CASE(HD_, W_)                                                                   \
  if (m.d == HD_ && m.W == W_)                                                                    \
    return bf ? launch_hash<HD_, W_, true>(X, R_dev, m.r, n_rows, seg_len, seg_stride, seg_off,   \
                                           out_stride, out_off, codes, st)                        \
              : launch_hash<HD_, W_, false>(X, R_dev, m.r, n_rows, seg_len, seg_stride, seg_off,  \
                                            out_stride, out_off, codes, st);
  LSHE_HASH_CASE(128, 1)
  LSHE_HASH_CASE(128, 2)
  LSHE_HASH_CASE(64, 1)
  LSHE_HASH_CASE(64, 2)
#undef LSHE_HASH_CASE
  return LSHE_UNSUPPORTED;
}

// ---- projection matrix to the device without a staging buffer --------------------------------
// The host values travel as kernel arguments (copied when the launch is enqueued, so the host
// array need not outlive the call and nothing is allocated or synchronised): each launch carries
// kProjChunk consecutive elements of the [d][r] matrix and stores them transposed, rounded to
// the compute type.
constexpr int kProjChunk = 960;   // floats per launch: 3840 bytes of the 4 KB argument block
struct ProjChunk {
  float v[kProjChunk];
};

template <bool BF16>
__global__ __launch_bounds__(256) void store_projection_kernel(const ProjChunk c, int first, int count,
                                                               int d, int r, void *R_dev) {
  for (int i = threadIdx.x; i < count; i += 256) {
    const int idx = first + i, row = idx / r, j = idx - row * r;   // element (row, j) of [d][r]
    const size_t o = (size_t)j * d + row;                          // -> hyperplane j, coordinate row
    if constexpr (BF16) ((uint16_t *)R_dev)[o] = (uint16_t)f32_to_bf16_bits(c.v[i]);
    else ((float *)R_dev)[o] = c.v[i];
  }
}

__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t *p, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace lshe

using namespace lshe;

extern "C" int lshe_init_projection(const lshe_config *cfg, uint64_t seed, const float *R_host,
                                    void *R_dev, void *stream) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (!R_dev) return LSHE_INVALID_ARG;
  const Dims m = dims_of(cfg);
  hipStream_t st = (hipStream_t)stream;
  const size_t bytes = (size_t)32 * m.Wr * m.d * m.esize;
  const long long words = (long long)(bytes / 4);
  // rows >= r stay zero
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                     (uint32_t *)R_dev, words);
  LSHE_HIP_TRY(hipGetLastError());
  const uint64_t key = splitmix64(seed);
  const int total = m.d * m.r;
  ProjChunk chunk;
  for (int first = 0; first < total; first += kProjChunk) {
    const int count = total - first < kProjChunk ? total - first : kProjChunk;
    for (int i = 0; i < count; ++i)
      chunk.v[i] = R_host ? R_host[first + i] : (float)normal_at(key, (uint64_t)(first + i));
    if (m.dtype == LSHE_BF16)
      hipLaunchKernelGGL((store_projection_kernel<true>), dim3(1), dim3(256), 0, st, chunk, first, count, m.d, m.r, R_dev);
    else
      hipLaunchKernelGGL((store_projection_kernel<false>), dim3(1), dim3(256), 0, st, chunk, first, count, m.d, m.r, R_dev);
    LSHE_HIP_TRY(hipGetLastError());
  }
  return LSHE_OK;
}

extern "C" int lshe_hash_keys(const lshe_config *cfg, const void *R_dev, const void *X, int64_t n,
                              uint32_t *codes, void *stream) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (n < 0) return LSHE_INVALID_ARG;
  if (n == 0) return LSHE_OK;
  if (!X || !codes || !R_dev) return LSHE_INVALID_ARG;
  Dims m = dims_of(cfg);
  m.W = m.Wr;   // eq. (2) whatever the eviction policy: ceil(r / 32) words per row
  return hash_rows(m, R_dev, X, n, n, n, 0, codes, (hipStream_t)stream);
}

extern "C" int lshe_key_norms(const lshe_config *cfg, const void *X, int64_t n, float *norm2,
                              void *stream) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  if (n < 0) return LSHE_INVALID_ARG;
  if (n == 0) return LSHE_OK;
  if (!X || !norm2) return LSHE_INVALID_ARG;
  return norm_rows(dims_of(cfg), X, n, (uint32_t *)norm2, (hipStream_t)stream);
}
