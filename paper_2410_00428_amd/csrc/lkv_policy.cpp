// Host-side policy of the layer-wise KV cache: the SLO-aware admission of prefills (paper Section 3.1,
// Eq. 1-3, Algorithm 1), the number of layers to retain so that a request's offload hides behind its
// prefill (Section 3.2.1, the offload-time model), the free-block forecast and the pressure rule
// (Section 3.2.1).  Pure functions of their arguments: no context, no device.
#include <cmath>
#include <cstdint>
#include <limits>

#include "lkv.h"

namespace {

bool bad_model(const lkv_cost_model *m) {
  return !m || m->num_layers <= 0 || m->head_dim <= 0 || m->num_heads <= 0 || !(m->device_flops > 0.0) ||
         !(m->link_bytes_per_s > 0.0) || !(m->bytes_per_elem > 0.0) || !(m->alpha >= 0.0) || !(m->beta >= 0.0) ||
         !(m->n_param >= 0.0) || !(m->n_hidden >= 0.0);
}

double prefill_seconds(const lkv_cost_model *m, int64_t seqlen) {
  const double s = (double)seqlen;
  return m->alpha * s * (2.0 * m->n_param + 2.0 * s * m->n_hidden) / m->device_flops;
}

double offload_seconds(const lkv_cost_model *m, int64_t seqlen, int32_t x) {
  return m->beta * (double)seqlen * 2.0 * (double)(m->num_layers - x) * (double)m->head_dim * (double)m->num_heads *
         m->bytes_per_elem / m->link_bytes_per_s;
}

// Tokens a decoding request is still expected to produce: the lower bound of its predicted length range minus
// what it has, never less than one.
int64_t tokens_to_come(const lkv_decode_request *r) {
  const int64_t left = r->predicted_lower_bound - r->n_past;
  return left > 1 ? left : 1;
}

double allow_seconds(const lkv_decode_request *r) {
  const double nf = (double)tokens_to_come(r);
  // the pace so far (waiting included); a request that has produced nothing is taken to run at its target
  const double tpot_now = r->n_past > 0 ? r->t_past / (double)r->n_past : r->t_tpot;
  return r->t_tpot * ((double)r->n_past + nf) - (r->t_past + tpot_now * nf);
}

}  // namespace

extern "C" {

double lkv_prefill_time(const lkv_cost_model *m, int64_t seqlen) {
  if (bad_model(m) || seqlen < 0) return std::numeric_limits<double>::quiet_NaN();
  return prefill_seconds(m, seqlen);
}

double lkv_offload_time(const lkv_cost_model *m, int64_t seqlen, int32_t x) {
  if (bad_model(m) || seqlen < 0 || x < 0 || x > m->num_layers) return std::numeric_limits<double>::quiet_NaN();
  return offload_seconds(m, seqlen, x);
}

lkv_status lkv_plan_offload(const lkv_cost_model *m, int64_t seqlen, int32_t *x_out, int32_t *retained_mask) {
  if (bad_model(m) || seqlen < 0 || !x_out) return LKV_ERR_INVALID_ARG;
  const double tp = prefill_seconds(m, seqlen);
  int32_t x = 0;
  while (x < m->num_layers && !(offload_seconds(m, seqlen, x) <= tp)) ++x;  // x = L offloads nothing: always fits
  *x_out = x;
  if (retained_mask) return lkv_plan_retained_layers(m->num_layers, x, retained_mask);
  return LKV_OK;
}

double lkv_allow_prefill_time(const lkv_decode_request *r) {
  if (!r || r->n_past < 0 || !(r->t_past >= 0.0) || !(r->t_tpot > 0.0)) return std::numeric_limits<double>::quiet_NaN();
  return allow_seconds(r);
}

lkv_status lkv_max_prefills(const lkv_decode_request *decoding, int32_t num_decoding, const double *prefill_times,
                            int32_t num_queued, int32_t *n_out) {
  if (num_decoding < 0 || num_queued < 0 || !n_out || (num_decoding && !decoding) || (num_queued && !prefill_times))
    return LKV_ERR_INVALID_ARG;
  double budget = std::numeric_limits<double>::infinity();  // nobody decoding: nothing constrains the queue
  for (int32_t i = 0; i < num_decoding; ++i) {
    const lkv_decode_request *r = decoding + i;
    if (r->n_past < 0 || !(r->t_past >= 0.0) || !(r->t_tpot > 0.0)) return LKV_ERR_INVALID_ARG;
    const double a = allow_seconds(r);
    if (a < budget) budget = a;
  }
  double total = 0.0;
  int32_t n = 0;
  while (n < num_queued) {
    if (!(prefill_times[n] >= 0.0)) return LKV_ERR_INVALID_ARG;
    total += prefill_times[n];
    if (!(total < budget)) break;  // strict, as in Algorithm 1
    ++n;
  }
  *n_out = n;
  return LKV_OK;
}

lkv_status lkv_forecast_avail(int64_t avail0, const int64_t *released, const int64_t *allocated, int32_t stages,
                              int64_t threshold, int64_t *avail_out, int32_t *first_below) {
  if (stages < 0 || (stages && (!released || !allocated))) return LKV_ERR_INVALID_ARG;
  int64_t a = avail0;
  int32_t first = -1;
  for (int32_t t = 0; t < stages; ++t) {
    a += released[t] - allocated[t];
    if (avail_out) avail_out[t] = a;
    if (first < 0 && a < threshold) first = t + 1;
  }
  if (first_below) *first_below = first;
  return LKV_OK;
}

lkv_status lkv_pressure_offload(int64_t deficit_blocks, const int32_t *retained, const int64_t *blocks_per_layer,
                                int32_t num_requests, int32_t *give) {
  if (num_requests < 0 || (num_requests && (!retained || !blocks_per_layer || !give))) return LKV_ERR_INVALID_ARG;
  for (int32_t r = 0; r < num_requests; ++r) {
    if (retained[r] < 0 || blocks_per_layer[r] < 0) return LKV_ERR_INVALID_ARG;
    give[r] = 0;
  }
  int64_t freed = 0;
  if (deficit_blocks <= 0) return LKV_OK;
  for (int32_t r = 0; r < num_requests && freed < deficit_blocks; ++r) {  // first pass: half, rounded up
    give[r] = (retained[r] + 1) / 2;
    freed += (int64_t)give[r] * blocks_per_layer[r];
  }
  for (int32_t r = 0; r < num_requests && freed < deficit_blocks; ++r) {  // second pass: the rest
    freed += (int64_t)(retained[r] - give[r]) * blocks_per_layer[r];
    give[r] = retained[r];
  }
  return LKV_OK;
}

}  // extern "C"
