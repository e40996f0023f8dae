// Host-only entry points: status strings, visible-context bookkeeping and the
// head classification of Dynamic Head Programming.  No GPU call is made here.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "df.h"

extern "C" const char *df_status_string(df_status s) {
  switch (s) {
    case DF_OK: return "ok";
    case DF_ERR_NULL: return "required pointer is NULL";
    case DF_ERR_SHAPE: return "non-positive or inconsistent size";
    case DF_ERR_UNSUPPORTED: return "unsupported head dim, head count, head type or mode";
    case DF_ERR_ALIGN: return "pointer or stride breaks 16-byte row alignment";
    case DF_ERR_WORKSPACE: return "workspace missing or too small";
    case DF_ERR_RANGE: return "offset, length or count out of range";
    case DF_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

// Sliding window of Sec. 3.1 with the per-type visibility of Eq. 2, 5 and 8.
extern "C" df_status df_head_context(int32_t head_type, int32_t T, int32_t sink_frames,
                                     int32_t window_frames, int32_t *n_sink, int32_t *n_win) {
  if (!n_sink || !n_win) return DF_ERR_NULL;
  if (T <= 0 || sink_frames < 0 || window_frames < 0) return DF_ERR_SHAPE;
  const int64_t s = int64_t(sink_frames) * T, w = int64_t(window_frames) * T;
  if (s > INT32_MAX || w > INT32_MAX) return DF_ERR_RANGE;
  switch (head_type) {
    case DF_HEAD_FULL: *n_sink = int32_t(s); *n_win = int32_t(w); break;
    case DF_HEAD_SINK: *n_sink = int32_t(s); *n_win = 0; break;
    case DF_HEAD_NEIGHBOR: *n_sink = 0; *n_win = int32_t(w); break;
    case DF_HEAD_DUMMY: *n_sink = 0; *n_win = 0; break;
    case DF_HEAD_PACK_DUMMY: *n_sink = 0; *n_win = T; break;
    default: return DF_ERR_UNSUPPORTED;
  }
  return DF_OK;
}

// Observation 1 (two-class) and the greedy rule that follows Eq. 7 (DHP).
// The sort key is formed in fp32, the precision the scores arrive in.
extern "C" df_status df_classify(const float *F, int32_t n, int32_t n_dummy, int32_t mode,
                                 uint8_t *type_out, float *key_out) {
  if (!F || !type_out) return DF_ERR_NULL;
  if (n <= 0) return DF_ERR_SHAPE;
  if (n_dummy < 0 || n_dummy > n) return DF_ERR_RANGE;
  if (mode != DF_CLASSIFY_TWO_CLASS && mode != DF_CLASSIFY_DHP) return DF_ERR_UNSUPPORTED;
  for (int64_t i = 0; i < int64_t(n) * 3; ++i)
    if (!std::isfinite(F[i])) return DF_ERR_RANGE;

  std::vector<float> key(n);
  for (int32_t h = 0; h < n; ++h) {
    const float f0 = F[3 * h], f1 = F[3 * h + 1];
    key[h] = (mode == DF_CLASSIFY_DHP) ? std::max(f0, f1) : f0 + f1;
  }
  std::vector<int32_t> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int32_t a, int32_t b) { return key[a] < key[b]; });
  for (int32_t h = 0; h < n; ++h) {
    if (mode == DF_CLASSIFY_TWO_CLASS) type_out[h] = DF_HEAD_FULL;
    else type_out[h] = (F[3 * h] >= F[3 * h + 1]) ? DF_HEAD_SINK : DF_HEAD_NEIGHBOR;
  }
  for (int32_t r = 0; r < n_dummy; ++r) type_out[order[r]] = DF_HEAD_DUMMY;
  if (key_out) std::copy(key.begin(), key.end(), key_out);
  return DF_OK;
}
