// Host-side planning for a change of parallel configuration: context overlap, device mapping
// (Kuhn-Munkres), migration order, cache discard, just-in-time arrangement, measured cost model.  No GPU.
#include <stdint.h>

#include <algorithm>
#include <limits>
#include <numeric>
#include <utility>
#include <iterator>
#include <vector>

#include "../../include/spotshard_plan.h"

namespace ss {
void set_error(const char *fmt, ...);
}
#define SS_FAIL(code, ...)        \
  do {                            \
    ::ss::set_error(__VA_ARGS__); \
    return (code);                \
  } while (0)

static int64_t overlap(int a0, int a1, int b0, int b1) { return std::max(0, std::min(a1, b1) - std::max(a0, b0)); }

static bool slice_ok(const ss_model_desc &m, const ss_slice &s) {
  return 0 <= s.layer_lo && s.layer_lo <= s.layer_hi && s.layer_hi <= m.n_layers && 0 <= s.head_lo &&
         s.head_lo <= s.head_hi && s.head_hi <= m.n_heads && 0 <= s.ffn_lo && s.ffn_lo <= s.ffn_hi && s.ffn_hi <= m.ffn;
}

extern "C" {

ss_status ss_context_overlap(const ss_model_desc *desc, int32_t lm_head_tied, const ss_slice *a, const ss_slice *b,
                             uint64_t kv_rows, uint64_t *model_bytes, uint64_t *cache_bytes) {
  if (!desc || !a || !b) SS_FAIL(SS_EINVAL, "NULL argument");
  const ss_model_desc &m = *desc;
  if (m.d_model < 1 || m.head_dim < 1 || m.vocab < 1 || !slice_ok(m, *a) || !slice_ok(m, *b))
    SS_FAIL(SS_EINVAL, "bad model descriptor or slice");
  const int64_t esz = m.dtype == SS_DTYPE_BF16 ? 2 : 4, kvsz = m.kv_dtype == SS_DTYPE_F32 ? 4 : 2;
  const int64_t d = m.d_model, Dh = m.head_dim;
  const int64_t layers = overlap(a->layer_lo, a->layer_hi, b->layer_lo, b->layer_hi);
  const int64_t heads = overlap(a->head_lo, a->head_hi, b->head_lo, b->head_hi);
  const int64_t ffn = overlap(a->ffn_lo, a->ffn_hi, b->ffn_lo, b->ffn_hi);
  const bool ln = m.norm == SS_NORM_LAYERNORM, glu = m.act == SS_ACT_SWIGLU, bias = m.has_bias != 0;
  // one layer: matrices in the weight type, vectors in float32
  int64_t per_layer = esz * (3 * d * heads * Dh + heads * Dh * d + (glu ? 2 : 1) * d * ffn + ffn * d);
  if (bias) per_layer += 4 * (3 * heads * Dh + (glu ? 0 : ffn));   // column-parallel biases follow their columns
  per_layer += 4 * ((ln ? 4 : 2) * d + (bias ? 2 * d : 0));        // norm gain (and shift) x2, the two row-parallel biases
  // replicated once per position: embedding, positions, LM head, final norm
  int64_t shared = esz * ((int64_t)m.vocab * d + (m.pos == SS_POS_LEARNED ? (int64_t)m.max_pos * d : 0) +
                          (lm_head_tied ? 0 : (int64_t)m.vocab * d)) +
                   4 * (ln ? 2 : 1) * d;
  if (model_bytes) *model_bytes = (uint64_t)(layers * per_layer + shared);
  if (cache_bytes) *cache_bytes = (uint64_t)(layers * 2 * heads * Dh * kvsz) * kv_rows;
  return SS_OK;
}

// Kuhn-Munkres in its potentials form on cost = max weight - weight (so a minimum-cost perfect
// matching is a maximum-weight one); rows are devices, columns positions; O(n^3).
ss_status ss_match_devices(int32_t n, const uint64_t *weight, int32_t *position_of, uint64_t *total) {
  if (n < 1 || n > 512 || !weight || !position_of) SS_FAIL(SS_EINVAL, "bad matching arguments");
  uint64_t wmax = 0;
  for (int64_t i = 0; i < (int64_t)n * n; ++i) wmax = std::max(wmax, weight[i]);
  if (wmax > (uint64_t)std::numeric_limits<int64_t>::max() / 4) SS_FAIL(SS_EINVAL, "weights too large");
  auto cost = [&](int u, int v) { return (int64_t)(wmax - weight[(size_t)u * n + v]); };
  const int64_t INF = std::numeric_limits<int64_t>::max() / 2;
  std::vector<int64_t> pu(n + 1, 0), pv(n + 1, 0), minv(n + 1);
  std::vector<int> row_of(n + 1, 0), way(n + 1, 0);  // row_of[col]: 1-based row matched to the column
  std::vector<char> used(n + 1);
  for (int u = 1; u <= n; ++u) {
    row_of[0] = u;
    int j0 = 0;
    std::fill(minv.begin(), minv.end(), INF);
    std::fill(used.begin(), used.end(), 0);
    do {
      used[j0] = 1;
      const int i0 = row_of[j0];
      int64_t delta = INF;
      int j1 = 0;
      for (int j = 1; j <= n; ++j) {
        if (used[j]) continue;
        const int64_t cur = cost(i0 - 1, j - 1) - pu[i0] - pv[j];
        if (cur < minv[j]) minv[j] = cur, way[j] = j0;
        if (minv[j] < delta) delta = minv[j], j1 = j;
      }
      for (int j = 0; j <= n; ++j) {
        if (used[j]) pu[row_of[j]] += delta, pv[j] -= delta;
        else minv[j] -= delta;
      }
      j0 = j1;
    } while (row_of[j0] != 0);
    do {
      const int j1 = way[j0];
      row_of[j0] = row_of[j1];
      j0 = j1;
    } while (j0);
  }
  uint64_t sum = 0;
  for (int j = 1; j <= n; ++j) {
    position_of[row_of[j] - 1] = j - 1;
    sum += weight[(size_t)(row_of[j] - 1) * n + (j - 1)];
  }
  if (total) *total = sum;
  return SS_OK;
}

ss_status ss_migration_order(int32_t n_layers, int32_t n_instances, const int64_t *delta, int64_t u_max,
                             int32_t *order) {
  if (n_layers < 1 || n_instances < 1 || !delta || !order) SS_FAIL(SS_EINVAL, "bad migration-order arguments");
  // usage[i]: instance i's buffer memory after the layers placed so far
  std::vector<int64_t> usage(n_instances, 0);
  auto peak_with = [&](int l) {
    const int64_t *d = delta + (size_t)l * n_instances;
    int64_t peak = usage[0] + d[0];
    for (int i = 1; i < n_instances; ++i) peak = std::max(peak, usage[i] + d[i]);
    return peak;
  };
  auto place = [&](int l) {
    const int64_t *d = delta + (size_t)l * n_instances;
    for (int i = 0; i < n_instances; ++i) usage[i] += d[i];
  };
  // The order is a partition of the layer list followed by a selection sort of its second part.
  // Front part: one in-order sweep keeps every layer that fits under u_max on top of the layers kept before it
  // (partition_copy visits its input once, front to back); the others are set aside in index order.
  std::vector<int32_t> all(n_layers), late;
  std::iota(all.begin(), all.end(), 0);
  late.reserve(n_layers);
  int32_t *front_end = std::partition_copy(all.begin(), all.end(), order, std::back_inserter(late), [&](int32_t l) {
                         if (peak_with(l) > u_max) return false;
                         place(l);
                         return true;
                       }).first;
  // Back part: of the layers set aside, always the one that leaves the lowest peak goes next (min_element takes the
  // first of equals, and rotating it to the front keeps the rest in index order: lowest index on ties).
  std::copy(late.begin(), late.end(), front_end);
  for (int32_t *next = front_end; next != order + n_layers; ++next) {
    int32_t *pick = std::min_element(next, order + n_layers, [&](int32_t a, int32_t b) { return peak_with(a) < peak_with(b); });
    std::rotate(next, pick, pick + 1);
    place(*next);
  }
  return SS_OK;
}

ss_status ss_progressive_plan(int32_t n_layers, const int32_t *order, const int32_t *stage_of_layer, int32_t n_stages,
                              int32_t *kind, int32_t *arg) {
  if (n_layers < 1 || n_stages < 1 || !order || !stage_of_layer || !kind || !arg) SS_FAIL(SS_EINVAL, "bad plan arguments");
  // A stage can start right after the slot of `order` in which the last of its layers arrives: find that slot
  // for every stage first, then write the plan out in one go.
  std::vector<int> slot_of_layer(n_layers, -1), last_slot(n_stages, -1);
  for (int i = 0; i < n_layers; ++i) {
    const int l = order[i];
    if (l < 0 || l >= n_layers || slot_of_layer[l] >= 0) SS_FAIL(SS_EINVAL, "order is not a permutation of the layers");
    slot_of_layer[l] = i;
  }
  for (int l = 0; l < n_layers; ++l) {
    const int p = stage_of_layer[l];
    if (p < 0 || p >= n_stages) SS_FAIL(SS_EINVAL, "layer %d has no stage", l);
    last_slot[p] = std::max(last_slot[p], slot_of_layer[l]);
  }
  for (int p = 0; p < n_stages; ++p)
    if (last_slot[p] < 0) SS_FAIL(SS_EINVAL, "stage %d has no layer", p);
  int k = 0;
  kind[k] = SS_PLAN_MIGRATE_CACHE, arg[k++] = -1;   // the cache context goes first
  for (int i = 0; i < n_layers; ++i) {
    const int p = stage_of_layer[order[i]];
    kind[k] = SS_PLAN_MIGRATE_LAYER, arg[k++] = order[i];
    if (last_slot[p] == i) kind[k] = SS_PLAN_START_STAGE, arg[k++] = p;
  }
  return SS_OK;
}

ss_status ss_rows_to_keep(int32_t n_rows, const int32_t *lens, int32_t keep, int32_t n_dst, int32_t *batch_map) {
  if (n_rows < 0 || keep < 0 || n_dst < 0 || (n_rows && !lens) || (n_dst && !batch_map)) SS_FAIL(SS_EINVAL, "bad arguments");
  std::vector<int> rows;
  for (int r = 0; r < n_rows; ++r) {
    if (lens[r] < 0) SS_FAIL(SS_EINVAL, "negative length");
    if (lens[r] > 0) rows.push_back(r);
  }
  std::stable_sort(rows.begin(), rows.end(), [&](int x, int y) { return lens[x] > lens[y]; });
  if ((int)rows.size() > std::min(keep, n_dst)) rows.resize(std::min(keep, n_dst));
  std::sort(rows.begin(), rows.end());
  for (int b = 0; b < n_dst; ++b) batch_map[b] = b < (int)rows.size() ? rows[b] : -1;
  return SS_OK;
}

int32_t ss_jit_iterations(int32_t acquisition, int32_t s_out, const double *l_exe, double t_grace, double t_mig) {
  if (s_out < 0 || !l_exe) return 0;
  int s = 0;
  if (!acquisition) {
    for (int k = 0; k <= s_out; ++k)
      if (l_exe[k] < t_grace - t_mig) s = k;
  } else {
    s = s_out;
    for (int k = 0; k <= s_out; ++k)
      if (l_exe[k] >= t_grace) {
        s = k;
        break;
      }
  }
  return t_mig < l_exe[s] ? s : 0;
}

// least-squares line y = c0 + c1 * x through the points; one distinct x: a constant (through_origin: c1 = y / x).
// non_decreasing: the best line among those with c1 >= 0, which is the constant through the mean when the
// unconstrained slope is negative.
static void fit_line(const std::vector<std::pair<double, double>> &pts, bool through_origin, bool non_decreasing, double *c0,
                     double *c1) {
  double mx = 0, my = 0;
  for (auto &p : pts) mx += p.first, my += p.second;
  mx /= (double)pts.size(), my /= (double)pts.size();
  double sxx = 0, sxy = 0;
  for (auto &p : pts) sxx += (p.first - mx) * (p.first - mx), sxy += (p.first - mx) * (p.second - my);
  if (sxx > 0 && !(non_decreasing && sxy < 0)) {
    *c1 = sxy / sxx, *c0 = my - *c1 * mx;
  } else if (sxx <= 0 && through_origin && mx > 0) {
    *c0 = 0, *c1 = my / mx;
  } else {
    *c0 = my, *c1 = 0;
  }
}

ss_status ss_cost_fit(const ss_cost_sample *decode, int32_t n_decode, const ss_cost_sample *prefill, int32_t n_prefill,
                      ss_cost_model *model) {
  if (!model || n_decode < 1 || !decode || n_prefill < 0 || (n_prefill && !prefill)) SS_FAIL(SS_EINVAL, "bad arguments");
  std::vector<int> batches;
  for (int i = 0; i < n_decode; ++i) {
    if (decode[i].batch < 1 || decode[i].length < 0 || !(decode[i].ms >= 0)) SS_FAIL(SS_EINVAL, "bad decode sample %d", i);
    batches.push_back(decode[i].batch);
  }
  std::sort(batches.begin(), batches.end());
  batches.erase(std::unique(batches.begin(), batches.end()), batches.end());
  if ((int)batches.size() > SS_COST_MAX_BATCHES) SS_FAIL(SS_EINVAL, "more than %d batch sizes", SS_COST_MAX_BATCHES);
  for (int i = 0; i < n_prefill; ++i) {
    if (prefill[i].length < 1 || !(prefill[i].ms >= 0)) SS_FAIL(SS_EINVAL, "bad initial-phase sample %d", i);
    if (!std::binary_search(batches.begin(), batches.end(), prefill[i].batch))
      SS_FAIL(SS_EINVAL, "initial-phase sample %d: batch size %d has no decode sample", i, prefill[i].batch);
  }
  *model = ss_cost_model{};
  model->n_batches = (int)batches.size();
  for (int b = 0; b < model->n_batches; ++b) {
    model->batch[b] = batches[b];
    std::vector<std::pair<double, double>> pts;
    for (int i = 0; i < n_decode; ++i)
      if (decode[i].batch == batches[b]) pts.push_back({(double)decode[i].length, decode[i].ms});
    fit_line(pts, false, true, &model->dec_base_ms[b], &model->dec_per_row_ms[b]);
    pts.clear();
    for (int i = 0; i < n_prefill; ++i)
      if (prefill[i].batch == batches[b]) pts.push_back({(double)prefill[i].length, prefill[i].ms});
    if (!pts.empty()) fit_line(pts, true, true, &model->pre_base_ms[b], &model->pre_per_token_ms[b]);
  }
  return SS_OK;
}

ss_status ss_cost_l_exe(const ss_cost_model *model, int32_t batch, int32_t s_in, int32_t s_out, double *l_exe) {
  if (!model || !l_exe || model->n_batches < 1 || model->n_batches > SS_COST_MAX_BATCHES || batch < 1 || s_in < 1 || s_out < 0)
    SS_FAIL(SS_EINVAL, "bad arguments");
  // the fitted batch sizes around `batch` and the weight of the upper one
  int hi = 0;
  while (hi < model->n_batches && model->batch[hi] < batch) ++hi;
  int lo = hi;
  double w = 0;
  if (hi == model->n_batches) {
    lo = hi = model->n_batches - 1;
  } else if (model->batch[hi] != batch && hi > 0) {
    lo = hi - 1;
    w = (double)(batch - model->batch[lo]) / (double)(model->batch[hi] - model->batch[lo]);
  }
  auto mix = [&](const double *base, const double *slope, double x) {
    return (1 - w) * (base[lo] + slope[lo] * x) + w * (base[hi] + slope[hi] * x);
  };
  l_exe[0] = mix(model->pre_base_ms, model->pre_per_token_ms, (double)s_in);
  for (int i = 1; i <= s_out; ++i)
    l_exe[i] = l_exe[i - 1] + mix(model->dec_base_ms, model->dec_per_row_ms, (double)(s_in + i - 1));
  return SS_OK;
}

}  // extern "C"
