// Chunked hand-off of activation payloads: two queues by phase, decode first, fixed-size prefill
// chunks, one device -> pinned-host copy at a time on the sender's own stream (paper section 4.2).
#include "../../include/molink_handoff.h"

#include <hip/hip_runtime.h>

#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

namespace {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

struct Item {
  int64_t ticket;
  int32_t kind;
  int64_t offset, bytes;
};

// Decode runs and prefill chunks of one payload, each in address order.
int split_payload(int32_t S, const int32_t* q_lens, int64_t row_bytes, int64_t chunk_bytes, std::vector<Item>* decode,
                  std::vector<Item>* prefill) {
  int64_t row = 0, run_start = -1;
  for (int s = 0; s < S; ++s) {
    const int64_t q = q_lens[s];
    if (q < 1) return fail(HANDOFF_ERR_ARG, "q_lens[%d] = %lld must be >= 1", s, (long long)q);
    if (q == 1) {
      if (run_start < 0) run_start = row;
    } else {
      if (run_start >= 0) {
        decode->push_back(Item{0, HANDOFF_DECODE, run_start * row_bytes, (row - run_start) * row_bytes});
        run_start = -1;
      }
      const int64_t end = (row + q) * row_bytes;
      for (int64_t off = row * row_bytes; off < end; off += chunk_bytes)
        prefill->push_back(Item{0, HANDOFF_PREFILL, off, end - off < chunk_bytes ? end - off : chunk_bytes});
    }
    row += q;
  }
  if (run_start >= 0) decode->push_back(Item{0, HANDOFF_DECODE, run_start * row_bytes, (row - run_start) * row_bytes});
  return HANDOFF_OK;
}

// A serving loop submits one payload per micro-batch for as long as it runs, so nothing here may grow with
// the number of payloads: a ticket's event and transfer lists are released as soon as its transfers are in the
// queues, finished tickets beyond the most recent kKeepTickets are forgotten (they read as complete), and the
// log keeps the most recent kMaxLog records.
constexpr size_t kKeepTickets = 4096;
constexpr size_t kMaxLog = 1 << 16;

struct Ticket {
  hipEvent_t ready;                     // nullptr once the ticket's transfers have been queued
  const char* dev;
  char* host;
  std::vector<Item> decode, prefill;
  int64_t left_decode, left_total;
  int64_t visible_pick;
  bool queued;
};

}  // namespace

struct handoff_sender {
  int device;
  int64_t chunk_bytes;
  hipStream_t stream;
  std::thread worker;
  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::deque<Ticket> tickets;           // tickets first_id, first_id + 1, ...
  int64_t first_id;                     // id of tickets.front(); older ones have completed and were forgotten
  size_t next_unqueued;                 // index in `tickets` of the first one whose transfers are not queued yet
  std::deque<Item> decode_q, prefill_q;
  std::deque<handoff_record> log;
  int64_t picks;
  bool stop, failed;
  char fail_msg[256];
  std::chrono::steady_clock::time_point t0;

  double now_ms() const {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  }

  // Move every ticket whose producer work has finished into the queues (in ticket order).
  // Called with the lock held.
  void admit_ready() {
    while (next_unqueued < tickets.size()) {
      Ticket& t = tickets[next_unqueued];
      if (hipEventQuery(t.ready) != hipSuccess) { (void)hipGetLastError(); break; }
      for (const Item& it : t.decode) decode_q.push_back(it);
      for (const Item& it : t.prefill) prefill_q.push_back(it);
      t.visible_pick = picks;
      t.queued = true;
      (void)hipEventDestroy(t.ready);
      t.ready = nullptr;
      std::vector<Item>().swap(t.decode);
      std::vector<Item>().swap(t.prefill);
      ++next_unqueued;
      cv_done.notify_all();             // a waiter on a kind this payload has no transfers of is done now
    }
  }

  Ticket& ticket_of(int64_t id) { return tickets[(size_t)(id - first_id)]; }

  // Forget finished tickets at the front beyond the ones kept for late queries.  Called with the lock held.
  void retire_old() {
    while (tickets.size() > kKeepTickets && next_unqueued > 0 && tickets.front().queued && tickets.front().left_total == 0) {
      tickets.pop_front();
      ++first_id;
      --next_unqueued;
    }
  }

  void record(const handoff_record& r) {
    if (log.size() >= kMaxLog) log.pop_front();
    log.push_back(r);
  }

  void run() {
    (void)hipSetDevice(device);
    std::unique_lock<std::mutex> lk(mu);
    for (;;) {
      admit_ready();
      if (decode_q.empty() && prefill_q.empty()) {
        if (next_unqueued < tickets.size()) {
          // a payload is still being produced: wait for it outside the lock
          hipEvent_t ev = tickets[next_unqueued].ready;
          lk.unlock();
          hipError_t e = hipEventSynchronize(ev);
          lk.lock();
          if (e != hipSuccess) { set_failed("hipEventSynchronize", e); }
          if (failed) { drop_everything(); }
          continue;
        }
        if (stop) return;
        cv_work.wait(lk);
        continue;
      }
      Item it;
      if (!decode_q.empty()) { it = decode_q.front(); decode_q.pop_front(); }
      else { it = prefill_q.front(); prefill_q.pop_front(); }
      const int64_t pick = picks++;
      const Ticket& t = ticket_of(it.ticket);
      const char* src = t.dev + it.offset;
      char* dst = t.host + it.offset;
      lk.unlock();
      const double begin = now_ms();
      hipError_t e = hipMemcpyAsync(dst, src, (size_t)it.bytes, hipMemcpyDeviceToHost, stream);
      if (e == hipSuccess) e = hipStreamSynchronize(stream);
      const double end = now_ms();
      lk.lock();
      if (e != hipSuccess) set_failed("device to host copy", e);
      record(handoff_record{it.ticket, it.kind, 0, it.offset, it.bytes, pick, begin, end});
      Ticket& tt = ticket_of(it.ticket);
      if (it.kind == HANDOFF_DECODE) --tt.left_decode;
      --tt.left_total;
      retire_old();
      cv_done.notify_all();
      if (failed) drop_everything();
    }
  }

  void set_failed(const char* what, hipError_t e) {
    if (!failed) snprintf(fail_msg, sizeof(fail_msg), "%s failed: %s", what, hipGetErrorString(e));
    failed = true;
  }

  // After a failed copy nothing more is moved; waiters are released with an error.
  void drop_everything() {
    decode_q.clear();
    prefill_q.clear();
    for (Ticket& t : tickets) {
      t.left_decode = 0; t.left_total = 0; t.queued = true;
      if (t.ready) { (void)hipEventDestroy(t.ready); t.ready = nullptr; }
    }
    next_unqueued = tickets.size();
    cv_done.notify_all();
  }
};

extern "C" {

int handoff_plan(int32_t num_seqs, const int32_t* q_lens, int64_t row_bytes, int64_t chunk_bytes, handoff_record* out,
                 int32_t capacity, int32_t* out_count) {
  if (!q_lens || !out_count || (!out && capacity > 0)) return fail(HANDOFF_ERR_NULL, "a required pointer is NULL");
  if (num_seqs < 1 || row_bytes < 1 || chunk_bytes < 1 || capacity < 0)
    return fail(HANDOFF_ERR_ARG, "num_seqs, row_bytes and chunk_bytes must be positive");
  std::vector<Item> d, p;
  int rc = split_payload(num_seqs, q_lens, row_bytes, chunk_bytes, &d, &p);
  if (rc) return rc;
  const size_t n = d.size() + p.size();
  *out_count = (int32_t)n;
  size_t k = 0;
  for (const std::vector<Item>* v : {&d, &p})
    for (const Item& it : *v) {
      if (k >= (size_t)capacity) return fail(HANDOFF_ERR_SIZE, "%zu records needed, room for %d", n, capacity);
      out[k++] = handoff_record{0, it.kind, 0, it.offset, it.bytes, 0, 0.0, 0.0};
    }
  return HANDOFF_OK;
}

int handoff_sender_create(int32_t device, int64_t chunk_bytes, handoff_sender** out) {
  if (!out) return fail(HANDOFF_ERR_NULL, "out pointer is NULL");
  *out = nullptr;
  if (chunk_bytes < 1) return fail(HANDOFF_ERR_ARG, "chunk_bytes must be positive");
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess) return fail(HANDOFF_ERR_HIP, "hipGetDeviceCount: %s", hipGetErrorString(e));
  if (device < 0 || device >= ndev) return fail(HANDOFF_ERR_ARG, "device %d outside [0, %d)", device, ndev);
  if ((e = hipSetDevice(device)) != hipSuccess) return fail(HANDOFF_ERR_HIP, "hipSetDevice: %s", hipGetErrorString(e));
  handoff_sender* s = new (std::nothrow) handoff_sender();
  if (!s) return fail(HANDOFF_ERR_ARG, "out of host memory");
  s->device = device;
  s->chunk_bytes = chunk_bytes;
  s->next_unqueued = 0;
  s->first_id = 0;
  s->picks = 0;
  s->stop = s->failed = false;
  s->fail_msg[0] = 0;
  s->t0 = std::chrono::steady_clock::now();
  if ((e = hipStreamCreateWithFlags(&s->stream, hipStreamNonBlocking)) != hipSuccess) {
    delete s;
    return fail(HANDOFF_ERR_HIP, "hipStreamCreateWithFlags: %s", hipGetErrorString(e));
  }
  s->worker = std::thread([s] { s->run(); });
  *out = s;
  return HANDOFF_OK;
}

int handoff_sender_submit(handoff_sender* s, void* producer_stream, const void* payload_dev, void* payload_host,
                          int32_t num_seqs, const int32_t* q_lens, int64_t row_bytes, int64_t* out_ticket) {
  if (!s || !payload_dev || !payload_host || !q_lens || !out_ticket)
    return fail(HANDOFF_ERR_NULL, "a required argument of handoff_sender_submit is NULL");
  if (num_seqs < 1 || row_bytes < 1) return fail(HANDOFF_ERR_ARG, "num_seqs and row_bytes must be positive");
  Ticket t;
  t.dev = (const char*)payload_dev;
  t.host = (char*)payload_host;
  int rc = split_payload(num_seqs, q_lens, row_bytes, s->chunk_bytes, &t.decode, &t.prefill);
  if (rc) return rc;
  hipError_t e = hipSetDevice(s->device);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&t.ready, hipEventDisableTiming);
  if (e != hipSuccess) return fail(HANDOFF_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
  if ((e = hipEventRecord(t.ready, (hipStream_t)producer_stream)) != hipSuccess) {
    (void)hipEventDestroy(t.ready);
    return fail(HANDOFF_ERR_HIP, "hipEventRecord: %s", hipGetErrorString(e));
  }
  t.left_decode = (int64_t)t.decode.size();
  t.left_total = (int64_t)(t.decode.size() + t.prefill.size());
  t.visible_pick = -1;
  t.queued = false;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->failed) {
      (void)hipEventDestroy(t.ready);
      return fail(HANDOFF_ERR_HIP, "the sender has failed: %s", s->fail_msg);
    }
    const int64_t id = s->first_id + (int64_t)s->tickets.size();
    for (Item& it : t.decode) it.ticket = id;
    for (Item& it : t.prefill) it.ticket = id;
    s->tickets.push_back(std::move(t));
    *out_ticket = id;
  }
  s->cv_work.notify_all();
  return HANDOFF_OK;
}

int handoff_sender_wait(handoff_sender* s, int64_t ticket, int32_t kind) {
  if (!s) return fail(HANDOFF_ERR_NULL, "sender is NULL");
  if (kind != HANDOFF_DECODE && kind != HANDOFF_PREFILL) return fail(HANDOFF_ERR_ARG, "unknown kind %d", kind);
  std::unique_lock<std::mutex> lk(s->mu);
  if (ticket < 0 || ticket >= s->first_id + (int64_t)s->tickets.size())
    return fail(HANDOFF_ERR_ARG, "unknown ticket %lld", (long long)ticket);
  s->cv_done.wait(lk, [&] {
    if (ticket < s->first_id) return true;          // finished long ago and forgotten
    const Ticket& t = s->ticket_of(ticket);
    return t.queued && (kind == HANDOFF_DECODE ? t.left_decode == 0 : t.left_total == 0);
  });
  if (s->failed) return fail(HANDOFF_ERR_HIP, "%s", s->fail_msg);
  return HANDOFF_OK;
}

int handoff_sender_visible_pick(handoff_sender* s, int64_t ticket, int64_t* out_pick) {
  if (!s || !out_pick) return fail(HANDOFF_ERR_NULL, "a required pointer is NULL");
  std::lock_guard<std::mutex> lk(s->mu);
  if (ticket < 0 || ticket >= s->first_id + (int64_t)s->tickets.size())
    return fail(HANDOFF_ERR_ARG, "unknown ticket %lld", (long long)ticket);
  if (ticket < s->first_id) return fail(HANDOFF_ERR_ARG, "ticket %lld finished too long ago to be remembered", (long long)ticket);
  *out_pick = s->ticket_of(ticket).visible_pick;
  return HANDOFF_OK;
}

int handoff_sender_picks(handoff_sender* s, int64_t* out_picks) {
  if (!s || !out_picks) return fail(HANDOFF_ERR_NULL, "a required pointer is NULL");
  std::lock_guard<std::mutex> lk(s->mu);
  *out_picks = s->picks;
  return HANDOFF_OK;
}

int handoff_sender_log(handoff_sender* s, handoff_record* out, int32_t capacity, int32_t* out_count) {
  if (!s || !out_count || (!out && capacity > 0)) return fail(HANDOFF_ERR_NULL, "a required pointer is NULL");
  std::lock_guard<std::mutex> lk(s->mu);
  *out_count = (int32_t)s->log.size();
  if ((size_t)capacity < s->log.size())
    return fail(HANDOFF_ERR_SIZE, "%zu records available, room for %d", s->log.size(), capacity);
  for (size_t i = 0; i < s->log.size(); ++i) out[i] = s->log[i];
  s->log.clear();
  return HANDOFF_OK;
}

void handoff_sender_destroy(handoff_sender* s) {
  if (!s) return;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    s->stop = true;
  }
  s->cv_work.notify_all();
  if (s->worker.joinable()) s->worker.join();
  (void)hipSetDevice(s->device);
  for (Ticket& t : s->tickets)
    if (t.ready) (void)hipEventDestroy(t.ready);
  (void)hipStreamDestroy(s->stream);
  delete s;
}

const char* handoff_last_error(void) { return g_error; }

}  // extern "C"
