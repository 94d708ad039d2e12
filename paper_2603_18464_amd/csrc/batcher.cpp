// Request queue of an Inference Worker with the dynamic-window trigger of Section 3.2, Eq. 1:
// a batch is released when the queue holds the target batch or the oldest request has waited T_max.
// Host code only; pushes may come from any thread (rollout workers), polls from the worker's thread.
#include <cmath>
#include <deque>
#include <limits>
#include <mutex>
#include <new>

#include "../../include/vla.h"

struct vla_batcher {
  int32_t target = 0;
  double t_max = 0.0;
  int64_t max_tokens = 0;
  std::mutex mu;
  std::deque<vla_request> q;
  double last_arrival = -std::numeric_limits<double>::infinity();
};

extern "C" {

int vla_batcher_create(int32_t target_batch, double t_max, int64_t max_tokens, vla_batcher** out) {
  if (!out) return VLA_E_NULL;
  *out = nullptr;
  if (target_batch <= 0 || !(t_max >= 0.0) || std::isinf(t_max) || max_tokens < 0) return VLA_E_CONFIG;
  vla_batcher* b = new (std::nothrow) vla_batcher();
  if (!b) return VLA_E_CAPACITY;
  b->target = target_batch;
  b->t_max = t_max;
  b->max_tokens = max_tokens;
  *out = b;
  return VLA_OK;
}

int vla_batcher_destroy(vla_batcher* b) {
  if (!b) return VLA_E_NULL;
  delete b;
  return VLA_OK;
}

int vla_batcher_push(vla_batcher* b, const vla_request* r) {
  if (!b || !r) return VLA_E_NULL;
  if (r->n_patches < 0 || r->n_instr < 0 || r->n_patches + (int64_t)r->n_instr < 1) return VLA_E_SHAPE;
  if (!(r->t_arrival == r->t_arrival)) return VLA_E_SHAPE;   // NaN
  std::lock_guard<std::mutex> lock(b->mu);
  if (b->max_tokens && r->n_patches + (int64_t)r->n_instr > b->max_tokens) return VLA_E_CAPACITY;
  vla_request c = *r;
  // The queue is first-in first-out and t_first is its head's arrival: a stamp taken before a racing
  // thread's earlier push got in must not make the head look younger than the requests behind it.
  if (c.t_arrival < b->last_arrival) c.t_arrival = b->last_arrival;
  b->last_arrival = c.t_arrival;
  b->q.push_back(c);
  return VLA_OK;
}

int vla_batcher_size(vla_batcher* b, int32_t* n) {
  if (!b || !n) return VLA_E_NULL;
  std::lock_guard<std::mutex> lock(b->mu);
  *n = (int32_t)b->q.size();
  return VLA_OK;
}

int vla_batcher_deadline(vla_batcher* b, double* t) {
  if (!b || !t) return VLA_E_NULL;
  std::lock_guard<std::mutex> lock(b->mu);
  *t = b->q.empty() ? std::numeric_limits<double>::infinity() : b->q.front().t_arrival + b->t_max;
  return VLA_OK;
}

int vla_batcher_poll(vla_batcher* b, double t_now, vla_request* out, int32_t cap, int32_t* n_out) {
  if (!b || !out || !n_out) return VLA_E_NULL;
  *n_out = 0;
  if (cap < 1) return VLA_E_CAPACITY;
  std::lock_guard<std::mutex> lock(b->mu);
  if (b->q.empty()) return VLA_OK;
  const bool full = (int64_t)b->q.size() >= b->target;
  const bool waited = t_now - b->q.front().t_arrival >= b->t_max;
  if (!full && !waited) return VLA_OK;
  int64_t tokens = 0;
  int32_t n = 0;
  const int32_t most = cap < b->target ? cap : b->target;   // e.g. the free cache slots of a continuous batcher
  while (!b->q.empty() && n < most) {
    const vla_request& r = b->q.front();
    const int64_t need = r.n_patches + (int64_t)r.n_instr;
    if (b->max_tokens && n > 0 && tokens + need > b->max_tokens) break;
    out[n++] = r;
    tokens += need;
    b->q.pop_front();
  }
  *n_out = n;
  return VLA_OK;
}

}  // extern "C"
