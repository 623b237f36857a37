// Adaptive batching scheduler (paper section 4.2, equations 2-5): per-function fill-or-expire queues whose ready
// batches are dispatched in order of deadline margin, and which emit the (adapter id, token count) arrays that the
// segment builder of the multi-LoRA layer consumes.  Host code only; the caller supplies the clock.
//
// Data structure: one ring-free FIFO (std::deque) per function; a poll touches every non-empty queue once
// (O(functions + dispatched requests)): at the scale of the paper (hundreds of functions per GPU) a decision takes
// microseconds, which bench.py reports.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <deque>
#include <new>
#include <vector>

#include "../../include/lora_sched.h"

namespace {

constexpr int32_t kMaxBatchLimit = 65536;  // requests one plan accepts

struct Request {
    int64_t id;
    double arrival;
    int32_t ntok;
};

struct Function {
    lora_function_profile prof;
    int32_t max_batch;   // B
    int32_t batch_size;  // N
    std::deque<Request> queue;
};

inline double t_batch(const lora_function_profile &p, int32_t b) { return p.t0_ms + p.alpha_ms * (double)(b - 1); }  // equation 2

// B: the largest b with T(b) <= slo (at least 1, at most the plan's limit and the profile's cap).  A closed form
// proposes, the defining predicate decides (floating point may put the quotient one off).
int32_t max_batch_of(const lora_function_profile &p) {
    int64_t b = 1;
    if (p.alpha_ms > 0.0) {
        const double q = floor((p.slo_ms - p.t0_ms) / p.alpha_ms) + 1.0;
        b = q < 1.0 ? 1 : (q > (double)kMaxBatchLimit ? kMaxBatchLimit : (int64_t)q);
    } else {
        b = p.t0_ms <= p.slo_ms ? kMaxBatchLimit : 1;
    }
    while (b < kMaxBatchLimit && t_batch(p, (int32_t)b + 1) <= p.slo_ms) ++b;
    while (b > 1 && t_batch(p, (int32_t)b) > p.slo_ms) --b;
    if (p.max_batch > 0 && b > p.max_batch) b = p.max_batch;
    return (int32_t)b;
}

inline bool finite_time(double t) { return t == t && t > -HUGE_VAL && t < HUGE_VAL; }

}  // namespace

struct lora_batcher {
    std::vector<Function> fn;
    int64_t next_id = 0;
    double last_time = -HUGE_VAL;
};

namespace {

struct Forming {
    int32_t function, n;
    double t_exp, margin, tb, w;
    bool ready;
};

// State of function i's forming batch at `now` with M batches sharing the GPU (false: queue empty).
bool forming(const lora_batcher *b, int32_t i, double now, int32_t M, Forming *out) {
    const Function &f = b->fn[i];
    if (f.queue.empty()) return false;
    const int32_t queued = (int32_t)std::min<size_t>(f.queue.size(), (size_t)f.batch_size);
    const double tb = t_batch(f.prof, queued);
    const double t_old = f.queue.front().arrival;
    const double delay = f.prof.slo_ms - t_batch(f.prof, f.batch_size);  // equation 3
    const double w = now - t_old;
    out->function = i;
    out->n = queued;
    out->tb = tb;
    out->w = w;
    out->t_exp = t_old + delay;
    out->margin = f.prof.slo_ms - (w + (double)M * tb);  // equations 4 and 5
    out->ready = queued == f.batch_size || now >= out->t_exp;
    return true;
}

}  // namespace

extern "C" {

int lora_batcher_create(lora_batcher **out, const lora_function_profile *functions, int32_t n_functions) {
    if (!out) return LORA_SCHED_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_functions < 0 || (n_functions > 0 && !functions)) return LORA_SCHED_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_functions; ++i) {
        const lora_function_profile &p = functions[i];
        if (!(p.t0_ms > 0.0) || !(p.alpha_ms >= 0.0) || !(p.slo_ms > 0.0) || !finite_time(p.t0_ms) || !finite_time(p.alpha_ms) ||
            !finite_time(p.slo_ms) || p.adapter < -1 || p.max_batch < 0)
            return LORA_SCHED_ERR_INVALID_ARG;
    }
    lora_batcher *b = new (std::nothrow) lora_batcher();
    if (!b) return LORA_SCHED_ERR_INVALID_ARG;
    b->fn.resize((size_t)n_functions);
    for (int32_t i = 0; i < n_functions; ++i) {
        b->fn[i].prof = functions[i];
        b->fn[i].max_batch = max_batch_of(functions[i]);
        b->fn[i].batch_size = std::max(1, b->fn[i].max_batch / 2);
    }
    *out = b;
    return LORA_SCHED_OK;
}

int lora_batcher_destroy(lora_batcher *b) {
    if (!b) return LORA_SCHED_ERR_INVALID_ARG;
    delete b;
    return LORA_SCHED_OK;
}

#define LORA_FN_CHECK(b, function)                                                                        \
    if (!(b) || (function) < 0 || (size_t)(function) >= (b)->fn.size()) return LORA_SCHED_ERR_INVALID_ARG

int lora_batcher_max_batch(const lora_batcher *b, int32_t function, int32_t *out) {
    LORA_FN_CHECK(b, function);
    if (!out) return LORA_SCHED_ERR_INVALID_ARG;
    *out = b->fn[function].max_batch;
    return LORA_SCHED_OK;
}

int lora_batcher_set_batch_size(lora_batcher *b, int32_t function, int32_t n) {
    LORA_FN_CHECK(b, function);
    if (n < 1 || n > b->fn[function].max_batch) return LORA_SCHED_ERR_INVALID_ARG;
    b->fn[function].batch_size = n;
    return LORA_SCHED_OK;
}

int lora_batcher_batch_size(const lora_batcher *b, int32_t function, int32_t *out) {
    LORA_FN_CHECK(b, function);
    if (!out) return LORA_SCHED_ERR_INVALID_ARG;
    *out = b->fn[function].batch_size;
    return LORA_SCHED_OK;
}

int lora_batcher_delay(const lora_batcher *b, int32_t function, double *delay_ms_out) {
    LORA_FN_CHECK(b, function);
    if (!delay_ms_out) return LORA_SCHED_ERR_INVALID_ARG;
    const Function &f = b->fn[function];
    *delay_ms_out = f.prof.slo_ms - t_batch(f.prof, f.batch_size);
    return LORA_SCHED_OK;
}

int lora_batcher_submit(lora_batcher *b, int32_t function, int32_t n_tokens, double now_ms, int64_t *request_id_out) {
    LORA_FN_CHECK(b, function);
    if (n_tokens < 0 || !finite_time(now_ms) || now_ms < b->last_time) return LORA_SCHED_ERR_INVALID_ARG;
    b->last_time = now_ms;
    const int64_t id = b->next_id++;
    b->fn[function].queue.push_back(Request{id, now_ms, n_tokens});
    if (request_id_out) *request_id_out = id;
    return LORA_SCHED_OK;
}

int lora_batcher_poll(lora_batcher *b, double now_ms, int32_t running, int32_t max_batches, lora_batch *batches,
                      int32_t max_requests, int64_t *request_ids, int32_t *req_adapter, int32_t *req_ntok,
                      int32_t *n_batches_out, int32_t *n_requests_out) {
    if (!b || !n_batches_out || !n_requests_out || running < 0 || max_batches < 0 || max_requests < 0 || !finite_time(now_ms))
        return LORA_SCHED_ERR_INVALID_ARG;
    if (max_batches > 0 && !batches) return LORA_SCHED_ERR_INVALID_ARG;
    if (max_requests > 0 && (!request_ids || !req_adapter || !req_ntok)) return LORA_SCHED_ERR_INVALID_ARG;
    *n_batches_out = 0;
    *n_requests_out = 0;
    const int32_t M = running + 1;
    std::vector<Forming> ready;
    for (int32_t i = 0; i < (int32_t)b->fn.size(); ++i) {
        Forming f;
        if (forming(b, i, now_ms, M, &f) && f.ready) ready.push_back(f);
    }
    std::sort(ready.begin(), ready.end(), [](const Forming &x, const Forming &y) {
        return x.margin < y.margin || (x.margin == y.margin && x.function < y.function);
    });
    int32_t nb = 0, nr = 0;
    bool blocked = false;
    for (const Forming &f : ready) {
        if (nb >= max_batches) break;
        if (nr + f.n > max_requests) {
            blocked = true;
            break;
        }
        Function &fn = b->fn[f.function];
        lora_batch &o = batches[nb];
        o.function = f.function;
        o.adapter = fn.prof.adapter;
        o.n = f.n;
        o.first = nr;
        o.wait_ms = f.w;
        o.margin_ms = f.margin;
        o.t_batch_ms = f.tb;
        for (int32_t k = 0; k < f.n; ++k) {
            const Request &r = fn.queue.front();
            request_ids[nr] = r.id;
            req_adapter[nr] = fn.prof.adapter;
            req_ntok[nr] = r.ntok;
            ++nr;
            fn.queue.pop_front();
        }
        ++nb;
    }
    *n_batches_out = nb;
    *n_requests_out = nr;
    return (blocked && nb == 0) ? LORA_SCHED_ERR_CAPACITY : LORA_SCHED_OK;
}

int lora_batcher_next_event(const lora_batcher *b, double now_ms, int32_t running, double *t_out) {
    if (!b || !t_out || running < 0 || !finite_time(now_ms)) return LORA_SCHED_ERR_INVALID_ARG;
    double t = HUGE_VAL;
    for (int32_t i = 0; i < (int32_t)b->fn.size(); ++i) {
        Forming f;
        if (!forming(b, i, now_ms, running + 1, &f)) continue;
        const double ti = f.n == b->fn[i].batch_size ? now_ms : std::max(now_ms, f.t_exp);
        t = std::min(t, ti);
    }
    *t_out = t;
    return LORA_SCHED_OK;
}

int lora_batcher_queued(const lora_batcher *b, int32_t function, int32_t *out) {
    LORA_FN_CHECK(b, function);
    if (!out) return LORA_SCHED_ERR_INVALID_ARG;
    *out = (int32_t)b->fn[function].queue.size();
    return LORA_SCHED_OK;
}

const char *lora_sched_strerror(int status) {
    switch (status) {
        case LORA_SCHED_OK:
            return "ok";
        case LORA_SCHED_ERR_INVALID_ARG:
            return "invalid argument";
        case LORA_SCHED_ERR_CAPACITY:
            return "output capacity too small, or not enough removable bytes";
        default:
            return "unknown status";
    }
}

}  // extern "C"
