/*
 * symb_batcher: host-side request queue in front of the segmented layer calls.
 *
 * Opportunistic batching (Sec. 3.7 "Opportunistic Batching", Sec. 3.6 "Independent Execution"):
 * clients move through the base model's layers independently; at each layer the executor may
 * wait a little to gather requests of several clients into one flattened batch (no padding:
 * token rows are simply concatenated).  How long a request may be held depends on its size:
 * a decode step of a few tokens waits briefly, a prefill or fine-tuning pass of thousands of
 * tokens can wait longer, because the wait is a small part of its own run time.  Latency-
 * sensitive (inference) requests are put first when a batch has to be cut at the token cap.
 *
 * Pure host logic, no GPU, no threads, no clock of its own: the caller passes the time.
 * The caller turns a formed batch (request ids in row order + segment offsets) into a
 * symb_batch for symb_base_linear_fwd / _bwd_input.  Plain C ABI, all pointers HOST.
 */
#ifndef SYMB_BATCHER_H
#define SYMB_BATCHER_H
#include <stdint.h>
#include "symb.h"
#ifdef __cplusplus
extern "C" {
#endif

typedef struct symb_batcher_ctx* symb_batcher;

typedef struct {
    int64_t id;                 /* caller's handle of the request (returned in batches) */
    int32_t client;             /* informational */
    int32_t n_tokens;           /* rows of this request at this layer, >= 1 */
    int32_t latency_sensitive;  /* 1 = inference request: goes first when a batch is cut */
    int32_t reserved;
    double arrival_us;          /* when it reached this layer's queue; non-decreasing per layer */
} symb_request;

/* A request may be held for  min(max_wait_us, base_wait_us + per_token_wait_us * n_tokens). */
typedef struct {
    double base_wait_us, per_token_wait_us, max_wait_us;
    int32_t max_tokens;         /* token cap of one batch; a single larger request still runs alone */
    int32_t reserved;
} symb_batch_policy;

symb_status symb_batcher_create(symb_batcher* out, const symb_batch_policy* policy, int32_t num_layers);
symb_status symb_batcher_destroy(symb_batcher b);

/* Appends a request to the queue of `layer`.  SYMB_ERR_INVALID_ARG on a bad layer, n_tokens < 1
 * or an arrival time earlier than the queue's last one. */
symb_status symb_batcher_submit(symb_batcher b, int32_t layer, const symb_request* r);

/* Number of queued requests / tokens of a layer. */
symb_status symb_batcher_pending(symb_batcher b, int32_t layer, int32_t* n_requests, int64_t* n_tokens);

/* The earliest time at which the layer's queue is due: the smallest arrival + allowed wait over
 * the queued requests, or the arrival of the request that fills the token cap, whichever is
 * earlier; +infinity for an empty queue. */
symb_status symb_batcher_next_due(symb_batcher b, int32_t layer, double* due_us);

/* If the queue is due at now_us, removes one batch from it and describes it: the latency-
 * sensitive requests in arrival order, then the others in arrival order, as many as fit under
 * the token cap (at least one).  ids_out[0..*n_out) and seg_offsets_out[0..*n_out] (row
 * offsets of the flattened batch, starting at 0) must have room for `capacity` / capacity + 1
 * entries; requests beyond `capacity` stay queued.  *n_out = 0 if nothing is due. */
symb_status symb_batcher_take(symb_batcher b, int32_t layer, double now_us, int32_t capacity,
                              int64_t* ids_out, int32_t* seg_offsets_out, int32_t* n_out);

#ifdef __cplusplus
}
#endif
#endif
