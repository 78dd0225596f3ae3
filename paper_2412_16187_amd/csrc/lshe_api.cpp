// Host-only helpers of the lshe C ABI.
#include "lshe_common.h"

using namespace lshe;

extern "C" const char *lshe_strerror(int status) {
  switch (status) {
    case LSHE_OK: return "ok";
    case LSHE_INVALID_ARG: return "invalid argument";
    case LSHE_UNSUPPORTED: return "unsupported shape";
    case LSHE_WORKSPACE_TOO_SMALL: return "workspace too small";
    case LSHE_HIP_ERROR: return "HIP runtime error";
    case LSHE_SCRATCH_EXCEEDED: return "configuration needs more than the built-in scratch array";
    default: return "unknown status";
  }
}

extern "C" const char *lshe_version(void) { return "lshe 0.1 (gfx950)"; }

extern "C" int lshe_check_config(const lshe_config *cfg) {
  int rc = validate(cfg);
  if (rc != LSHE_OK) return rc;
  const int G = cfg->gqa_group;
  if (G != 1 && G != 2 && G != 4 && G != 8) return LSHE_UNSUPPORTED;
  return LSHE_OK;
}

extern "C" size_t lshe_projection_bytes(const lshe_config *cfg) {
  if (validate(cfg) != LSHE_OK) return 0;
  const Dims m = dims_of(cfg);
  return (size_t)32 * m.Wr * m.d * m.esize;
}

extern "C" size_t lshe_code_cache_bytes(const lshe_config *cfg) {
  if (validate(cfg) != LSHE_OK) return 0;
  const Dims m = dims_of(cfg);
  return (size_t)m.units * m.C * m.W * 4;
}

extern "C" const char *lshe_decode_plan(const lshe_config *cfg) {
  if (lshe_check_config(cfg) != LSHE_OK) return nullptr;
  const Dims m = dims_of(cfg);
  if (decode_is_fused(m.units, m.C, m.G))
    return fused_select_is_solo(m) ? "decode_fused_solo_kernel" : "decode_fused_kernel";
  const int S = attn_splits(m.units, m.C);
  if (S > 1) return S <= kMergeSmallRanges ? "attn_local_kernel + merge_small_kernel" : "attn_local_kernel + merge_local_kernel";
  return "select_kernel + attn_kernel";
}

extern "C" size_t lshe_workspace_bytes(const lshe_config *cfg, int32_t n_prompt) {
  if (validate(cfg) != LSHE_OK || n_prompt < 0) return 0;
  const Dims m = dims_of(cfg);
  const size_t a = decode_ws_bytes(m), b = prefill_ws_bytes(m, n_prompt);
  return a > b ? a : b;
}
