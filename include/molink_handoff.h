/*
 * Chunked hand-off of a stage's activation payload (paper section 4.2, "Chunk Transmission").
 *
 * A stage's output is one activation row per processed token, so a prefill request hands over up
 * to a thousand times more bytes than a decode request, and a decode payload that becomes ready
 * while a prefill payload is on the wire waits behind it.  The method: finished requests' volumes
 * go into two queues by phase, the sender always serves the decode queue first, and prefill
 * volumes are cut into chunks of a fixed size, so a decode volume waits for at most the one
 * chunk that is on the wire when it becomes ready.
 *
 * Here the wire is the copy engine: transfers are device -> pinned host copies on the sender's own
 * stream (default priority), issued one at a time by a worker thread, so they overlap with the
 * kernels of the next stage_forward.  A micro-batch is visible to the sender once the work that
 * was in its producer stream at submission has finished.  Layout of a payload: rows packed
 * sequence after sequence (stage_forward's hidden_out); a sequence with q_len 1 is a decode
 * request, with more a prefill request; consecutive decode rows form one transfer; every prefill
 * request's span is chunked on its own, chunks in address order, the last one shorter; each queue
 * is first-in first-out across micro-batches.  A transfer copies payload_dev[offset, offset+bytes)
 * to payload_host[offset, offset+bytes).
 *
 * Every entry point returns 0 or a negative HANDOFF_ERR_* code and never throws.
 */
#ifndef MOLINK_HANDOFF_H
#define MOLINK_HANDOFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  HANDOFF_OK = 0,
  HANDOFF_ERR_NULL = -1,   /* a required pointer is NULL */
  HANDOFF_ERR_ARG = -2,    /* a size or length is not positive, or a ticket is unknown */
  HANDOFF_ERR_SIZE = -3,   /* the caller's record array is too small (out_count has the need) */
  HANDOFF_ERR_HIP = -4     /* a HIP runtime call failed (also reported by waits when a copy failed) */
};

enum { HANDOFF_DECODE = 0, HANDOFF_PREFILL = 1 };

typedef struct {
  int64_t ticket;      /* micro-batch the transfer belongs to (0 for handoff_plan) */
  int32_t kind;        /* HANDOFF_DECODE or HANDOFF_PREFILL */
  int32_t reserved;
  int64_t offset;      /* byte offset in the payload */
  int64_t bytes;
  int64_t pick;        /* position in the sender's order of transfers (0 for handoff_plan) */
  double begin_ms;     /* host clock, ms since the sender was created: copy issued / copy finished */
  double end_ms;
} handoff_record;

typedef struct handoff_sender handoff_sender;

/*
 * Host only: the transfers of one micro-batch, decode runs first, then prefill chunks, each in
 * address order.  num_seqs > 0, q_lens[s] >= 1 host int32, row_bytes > 0, chunk_bytes > 0.
 * Writes at most `capacity` records; *out_count receives the number the payload has.
 */
int handoff_plan(int32_t num_seqs, const int32_t *q_lens, int64_t row_bytes, int64_t chunk_bytes,
                 handoff_record *out, int32_t capacity, int32_t *out_count);

/* A sender with its own stream and worker thread on HIP device `device`. */
int handoff_sender_create(int32_t device, int64_t chunk_bytes, handoff_sender **out);

/*
 * Hand a micro-batch's payload to the sender.  producer_stream (hipStream_t, NULL = default
 * stream): the payload is complete once the work now in this stream has finished; the call records
 * an event there and returns at once.  payload_dev: device memory, payload_host: pinned host
 * memory, both of sum(q_lens) * row_bytes bytes, both owned by the caller and left alone by it
 * until handoff_sender_wait(ticket, HANDOFF_PREFILL) has returned.  q_lens is copied.
 * *out_ticket receives the micro-batch's ticket (0, 1, 2, ... in submission order).
 */
int handoff_sender_submit(handoff_sender *s, void *producer_stream, const void *payload_dev, void *payload_host,
                          int32_t num_seqs, const int32_t *q_lens, int64_t row_bytes, int64_t *out_ticket);

/* Block until the ticket's decode transfers (kind = HANDOFF_DECODE) or all of its transfers
 * (HANDOFF_PREFILL) have finished. */
int handoff_sender_wait(handoff_sender *s, int64_t ticket, int32_t kind);

/* How many transfers the sender had chosen when it first saw the ticket complete (-1: not seen yet).
 * The sender remembers the 4096 most recent tickets; an older, finished one is HANDOFF_ERR_ARG here and
 * reads as complete in handoff_sender_wait. */
int handoff_sender_visible_pick(handoff_sender *s, int64_t ticket, int64_t *out_pick);

/* How many transfers the sender has chosen so far (its position in the order of transfers). */
int handoff_sender_picks(handoff_sender *s, int64_t *out_picks);

/* Copy out (and forget) the records of the transfers finished so far, in the order they were chosen.
 * The sender keeps at most the 65536 most recent records between two calls; older ones are dropped. */
int handoff_sender_log(handoff_sender *s, handoff_record *out, int32_t capacity, int32_t *out_count);

/* Finish the queued transfers, stop the worker, release the stream. */
void handoff_sender_destroy(handoff_sender *s);

/* Message describing the calling thread's most recent error ("" if none). */
const char *handoff_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
