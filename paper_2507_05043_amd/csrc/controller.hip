// Micro-batch count of a pipeline iteration from the stages' start-up latency profiles and the
// monitored links (paper section 4.1).  Host code only.
#include "../../include/molink_controller.h"

#include <cstdarg>
#include <cstdio>

namespace {

thread_local char g_error[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

// Latency of a stage at micro-batch size b: linear interpolation in the profile, constant below its
// first point, the last segment's slope beyond its last.
double latency_at(const mbc_stage_profile& p, int b) {
  const mbc_point* pt = p.points;
  const int n = p.num_points;
  if (b <= pt[0].batch || n == 1) return pt[0].ms;
  int i = 1;
  while (i < n - 1 && b > pt[i].batch) ++i;
  const double x0 = pt[i - 1].batch, x1 = pt[i].batch;
  return pt[i - 1].ms + (pt[i].ms - pt[i - 1].ms) * ((double)b - x0) / (x1 - x0);
}

int check(int32_t num_stages, const mbc_stage_profile* stages, const mbc_link* links, int32_t num_seqs,
          double act_bytes, double tok_bytes, const mbc_choice* out) {
  if (!stages || !links || !out) return fail(MBC_ERR_NULL, "a required pointer is NULL");
  if (num_stages < 1 || num_seqs < 1) return fail(MBC_ERR_ARG, "num_stages and num_seqs must be positive");
  if (!(act_bytes >= 0.0) || !(tok_bytes >= 0.0)) return fail(MBC_ERR_ARG, "payload sizes must be non-negative");
  for (int p = 0; p < num_stages; ++p) {
    if (!stages[p].points || stages[p].num_points < 1) return fail(MBC_ERR_ARG, "stage %d has no profile", p);
    for (int i = 0; i < stages[p].num_points; ++i) {
      if (stages[p].points[i].batch < 1 || !(stages[p].points[i].ms > 0.0))
        return fail(MBC_ERR_ARG, "stage %d: profile point %d must have batch >= 1 and a positive latency", p, i);
      if (i > 0 && stages[p].points[i].batch <= stages[p].points[i - 1].batch)
        return fail(MBC_ERR_ARG, "stage %d: profile points must ascend in batch", p);
    }
    if (!(links[p].latency_ms >= 0.0) || !(links[p].bytes_per_ms > 0.0))
      return fail(MBC_ERR_ARG, "link %d needs latency >= 0 and bandwidth > 0", p);
  }
  return MBC_OK;
}

mbc_choice evaluate(int32_t num_stages, const mbc_stage_profile* stages, const mbc_link* links, int32_t num_seqs,
                    double act_bytes, double tok_bytes, int32_t n) {
  mbc_choice c;
  c.num_microbatches = n;
  c.batch_per_microbatch = (num_seqs + n - 1) / n;
  double round_trip = 0.0, busiest = 0.0;
  for (int p = 0; p < num_stages; ++p) {
    const double compute = latency_at(stages[p], c.batch_per_microbatch);
    const double bytes = (p == num_stages - 1 ? tok_bytes : act_bytes) * c.batch_per_microbatch;
    const double serial = bytes / links[p].bytes_per_ms;
    round_trip += compute + serial + links[p].latency_ms;
    if (compute > busiest) busiest = compute;
    if (serial > busiest) busiest = serial;
  }
  c.round_trip_ms = round_trip;
  c.busiest_ms = n * busiest;
  c.period_ms = round_trip > c.busiest_ms ? round_trip : c.busiest_ms;
  return c;
}

}  // namespace

extern "C" {

int mbc_evaluate(int32_t num_stages, const mbc_stage_profile* stages, const mbc_link* links, int32_t num_seqs,
                 double activation_bytes_per_seq, double token_bytes_per_seq, int32_t num_microbatches,
                 mbc_choice* out) {
  int rc = check(num_stages, stages, links, num_seqs, activation_bytes_per_seq, token_bytes_per_seq, out);
  if (rc) return rc;
  if (num_microbatches < 1 || num_microbatches > num_seqs)
    return fail(MBC_ERR_ARG, "num_microbatches %d outside [1, num_seqs=%d]", num_microbatches, num_seqs);
  *out = evaluate(num_stages, stages, links, num_seqs, activation_bytes_per_seq, token_bytes_per_seq, num_microbatches);
  return MBC_OK;
}

int mbc_choose(int32_t num_stages, const mbc_stage_profile* stages, const mbc_link* links, int32_t num_seqs,
               double activation_bytes_per_seq, double token_bytes_per_seq, int32_t max_batch_per_microbatch,
               int32_t max_microbatches, mbc_choice* out) {
  int rc = check(num_stages, stages, links, num_seqs, activation_bytes_per_seq, token_bytes_per_seq, out);
  if (rc) return rc;
  if (max_microbatches < 1) return fail(MBC_ERR_ARG, "max_microbatches must be positive");
  const int n_max = max_microbatches < num_seqs ? max_microbatches : num_seqs;
  int n = max_batch_per_microbatch > 0 ? (num_seqs + max_batch_per_microbatch - 1) / max_batch_per_microbatch : 1;
  if (n > n_max)
    return fail(MBC_ERR_ARG, "%d sequences in micro-batches of at most %d need %d micro-batches, more than %d allowed",
                num_seqs, max_batch_per_microbatch, n, n_max);
  // The search goes on for as long as bubbles remain - the busiest stage or link still idles between micro-batches,
  // N * busiest < round trip - because a further micro-batch's work can then be hidden in them.  Comparing N + 1
  // with N alone would stall on the plateaus of ceil(num_seqs / N): from about sqrt(num_seqs) on, consecutive
  // counts give the same micro-batch size and the same round trip while bubbles are still there.  Among the counts
  // visited the shortest modelled iteration wins, the smallest count among equals.
  mbc_choice cur = evaluate(num_stages, stages, links, num_seqs, activation_bytes_per_seq, token_bytes_per_seq, n);
  mbc_choice best = cur;
  while (n < n_max && cur.busiest_ms < cur.round_trip_ms) {
    ++n;
    cur = evaluate(num_stages, stages, links, num_seqs, activation_bytes_per_seq, token_bytes_per_seq, n);
    if (cur.period_ms < best.period_ms) best = cur;
  }
  *out = best;
  return MBC_OK;
}

const char* mbc_last_error(void) { return g_error; }

}  // extern "C"
