/*
 * Micro-batch count for one iteration of a pipeline of inference engines (paper section 4.1,
 * "Dynamic Micro-batch").  Host only.
 *
 * When the links between the engines are slow, a pipeline run with as many micro-batches as it has
 * stages idles: a stage that has finished its micro-batches waits for the next one to arrive.  More
 * micro-batches fill those bubbles until the busiest stage (or link) has no idle time left.  The head
 * engine's controller therefore combines (1) the latency table every engine measured at start-up
 * (computation latency over micro-batch sizes) with (2) the monitored latency and bandwidth of every
 * link, caps the micro-batch size, and searches the micro-batch count N upwards from the smallest
 * admissible one for as long as bubbles remain in which a further micro-batch's computation can hide.
 *
 * The model behind the search: all N micro-batches hold b = ceil(num_seqs / N) sequences; stage p
 * needs c_p(b) per micro-batch (linear interpolation in the profile, constant below its first point,
 * the last segment's slope beyond its last); link p (stage p -> p+1, the last link back to the head)
 * is occupied s_p(b) = bytes / bandwidth per micro-batch and adds its latency on top.  One iteration
 * then takes
 *     period(N) = max( round trip = sum_p c_p + s_p + latency_p ,  N * max_p max(c_p, s_p) ),
 * the first term while bubbles remain, the second once the busiest resource is saturated.
 *
 * Every entry point returns 0 or a negative MBC_ERR_* code and never throws.
 */
#ifndef MOLINK_CONTROLLER_H
#define MOLINK_CONTROLLER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MBC_OK = 0, MBC_ERR_NULL = -1, MBC_ERR_ARG = -2 };

typedef struct {
  int32_t batch;   /* sequences in the micro-batch */
  double ms;       /* measured computation latency of the stage */
} mbc_point;

typedef struct {
  const mbc_point *points;   /* ascending in batch, at least one */
  int32_t num_points;
} mbc_stage_profile;

typedef struct {
  double latency_ms;     /* >= 0 */
  double bytes_per_ms;   /* > 0 */
} mbc_link;

typedef struct {
  int32_t num_microbatches;       /* N */
  int32_t batch_per_microbatch;   /* b = ceil(num_seqs / N) */
  double period_ms;               /* modelled time of one iteration */
  double round_trip_ms;           /* first term of the maximum */
  double busiest_ms;              /* second term of the maximum */
} mbc_choice;

/*
 * Modelled iteration for a given N.  stages: num_stages profiles; links: num_stages links (the payload
 * of link p < num_stages-1 is activation_bytes_per_seq per sequence, of the last link
 * token_bytes_per_seq).  1 <= num_microbatches <= num_seqs.
 */
int mbc_evaluate(int32_t num_stages, const mbc_stage_profile *stages, const mbc_link *links, int32_t num_seqs,
                 double activation_bytes_per_seq, double token_bytes_per_seq, int32_t num_microbatches,
                 mbc_choice *out);

/*
 * The controller's choice: N runs upwards from ceil(num_seqs / max_batch_per_microbatch) (the cap on
 * the micro-batch size; <= 0 = no cap, N starts at 1) for as long as bubbles remain at N, i.e. while
 * N * max_p max(c_p, s_p) < round trip, and stops at the first N whose busiest stage or link has no idle
 * time left, or at min(max_microbatches, num_seqs).  The choice is the visited N with the shortest modelled
 * iteration, the smallest such N among equals (counts that give the same micro-batch size also give the same
 * round trip, so a step from N to N + 1 alone says nothing while bubbles remain).
 */
int mbc_choose(int32_t num_stages, const mbc_stage_profile *stages, const mbc_link *links, int32_t num_seqs,
               double activation_bytes_per_seq, double token_bytes_per_seq, int32_t max_batch_per_microbatch,
               int32_t max_microbatches, mbc_choice *out);

/* Message describing the calling thread's most recent error ("" if none). */
const char *mbc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
