// Host-side opportunistic batching queue (see include/symb_batcher.h).  No device code.
#include "../../include/symb_batcher.h"

#include <algorithm>
#include <cmath>
#include <deque>
#include <limits>
#include <new>
#include <vector>

struct symb_batcher_ctx {
    symb_batch_policy policy;
    std::vector<std::deque<symb_request>> queues;
};

namespace {

double allowed_wait(const symb_batch_policy& p, int32_t n_tokens) {
    return std::min(p.max_wait_us, p.base_wait_us + p.per_token_wait_us * (double)n_tokens);
}

// Smallest arrival + allowed wait, or the arrival that brings the queued tokens to the cap.
double due_time(const symb_batch_policy& p, const std::deque<symb_request>& q) {
    double due = std::numeric_limits<double>::infinity();
    int64_t tokens = 0;
    for (const symb_request& r : q) {
        due = std::min(due, r.arrival_us + allowed_wait(p, r.n_tokens));
        tokens += r.n_tokens;
        if (tokens >= p.max_tokens) {
            due = std::min(due, r.arrival_us);
            break;
        }
    }
    return due;
}

bool bad_policy(const symb_batch_policy* p) {
    return !p || !(p->base_wait_us >= 0) || !(p->per_token_wait_us >= 0) || !(p->max_wait_us >= 0) || p->max_tokens < 1;
}

}  // namespace

extern "C" {

symb_status symb_batcher_create(symb_batcher* out, const symb_batch_policy* policy, int32_t num_layers) {
    if (!out || bad_policy(policy) || num_layers < 1) return SYMB_ERR_INVALID_ARG;
    symb_batcher_ctx* c = new (std::nothrow) symb_batcher_ctx;
    if (!c) return SYMB_ERR_DEVICE;
    c->policy = *policy;
    c->queues.resize((size_t)num_layers);
    *out = c;
    return SYMB_OK;
}

symb_status symb_batcher_destroy(symb_batcher b) {
    delete b;
    return SYMB_OK;
}

symb_status symb_batcher_submit(symb_batcher b, int32_t layer, const symb_request* r) {
    if (!b || !r || layer < 0 || layer >= (int32_t)b->queues.size() || r->n_tokens < 1 || !std::isfinite(r->arrival_us))
        return SYMB_ERR_INVALID_ARG;
    std::deque<symb_request>& q = b->queues[(size_t)layer];
    if (!q.empty() && r->arrival_us < q.back().arrival_us) return SYMB_ERR_INVALID_ARG;
    q.push_back(*r);
    return SYMB_OK;
}

symb_status symb_batcher_pending(symb_batcher b, int32_t layer, int32_t* n_requests, int64_t* n_tokens) {
    if (!b || layer < 0 || layer >= (int32_t)b->queues.size()) return SYMB_ERR_INVALID_ARG;
    int64_t t = 0;
    for (const symb_request& r : b->queues[(size_t)layer]) t += r.n_tokens;
    if (n_requests) *n_requests = (int32_t)b->queues[(size_t)layer].size();
    if (n_tokens) *n_tokens = t;
    return SYMB_OK;
}

symb_status symb_batcher_next_due(symb_batcher b, int32_t layer, double* due_us) {
    if (!b || !due_us || layer < 0 || layer >= (int32_t)b->queues.size()) return SYMB_ERR_INVALID_ARG;
    *due_us = due_time(b->policy, b->queues[(size_t)layer]);
    return SYMB_OK;
}

symb_status symb_batcher_take(symb_batcher b, int32_t layer, double now_us, int32_t capacity, int64_t* ids_out,
                              int32_t* seg_offsets_out, int32_t* n_out) {
    if (!b || !ids_out || !seg_offsets_out || !n_out || capacity < 1 || layer < 0 || layer >= (int32_t)b->queues.size())
        return SYMB_ERR_INVALID_ARG;
    std::deque<symb_request>& q = b->queues[(size_t)layer];
    *n_out = 0;
    seg_offsets_out[0] = 0;
    if (q.empty() || due_time(b->policy, q) > now_us) return SYMB_OK;
    // candidates: what has arrived by now; latency-sensitive first, arrival order inside each class
    std::vector<size_t> order;
    for (int cls = 1; cls >= 0; --cls)
        for (size_t i = 0; i < q.size(); ++i)
            if (q[i].arrival_us <= now_us && (q[i].latency_sensitive != 0) == (cls == 1)) order.push_back(i);
    std::vector<char> taken(q.size(), 0);
    int64_t tokens = 0;
    int32_t n = 0;
    for (size_t i : order) {
        if (n == capacity) break;
        if (n > 0 && tokens + q[i].n_tokens > b->policy.max_tokens) continue;   // does not fit: stays for the next batch
        ids_out[n] = q[i].id;
        tokens += q[i].n_tokens;
        seg_offsets_out[n + 1] = (int32_t)tokens;
        taken[i] = 1;
        ++n;
    }
    std::deque<symb_request> rest;
    for (size_t i = 0; i < q.size(); ++i)
        if (!taken[i]) rest.push_back(q[i]);
    q.swap(rest);
    *n_out = n;
    return SYMB_OK;
}

}  // extern "C"
