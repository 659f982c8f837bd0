/*
 * lemix_serve.h - the continuous-batching loop of one stage (Autoregressive
 * Generation, Algorithm 3): requests are batched FCFS up to C with the
 * waiting limit T_w, every pass runs ONE hybrid iteration-level mini-batch
 * (the ongoing decodes plus newly admitted prompt chunks) through stage_step,
 * and finished requests leave the batch.
 *
 * The server owns what the loop needs beyond the stage: the batcher, the page
 * allocator over the caller's KV pool (a free list; a request holds
 * ceil(tokens / page_size) pages and returns them when it finishes; it starts
 * only once the pages of its whole sequence can be set aside, so every started
 * request runs to its end and the loop always drains), the
 * per-request progress, and small device buffers allocated in
 * ls_server_create (the batch's X and Y rows, block table, context lengths,
 * row pointers) and freed in ls_server_destroy.
 *
 * A mid-pipeline stage receives every token's input row from the stage before
 * it and produces the row for the stage after it; a request therefore brings
 * X [dev] [prompt_len + n_decode, d] (the prompt rows, then the input row of
 * each decode step) and Y [dev] of the same shape, both io_dtype and owned by
 * the caller until the request is reported finished and the stream has
 * drained.
 *
 * Calls enqueue work on `stream` and do not synchronise, except that a pass
 * waits for the host-to-device copy of the pass two before it (its staging
 * slot is reused).  Every pass of one server must use the same stream: pages
 * freed by one pass are handed out again by later ones, and stream order is
 * what keeps those uses apart.  One owner thread per server.  Training tasks
 * do not go through the server (Algorithm 2's loop, ls_node_execute, runs
 * them).
 */
#ifndef LEMIX_SERVE_H
#define LEMIX_SERVE_H

#include "lemix_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ls_server ls_server; /* opaque */

typedef struct {
  int32_t max_batch;         /* C of Algorithm 3: requests per mini-batch, 1..256 */
  double max_wait;           /* T_w of Algorithm 3, seconds on the caller's clock */
  int32_t n_pages;           /* pages in k_pool / v_pool; the server hands out all of them */
  int32_t max_pages_per_req; /* block-table row length; a request holds at most this many pages */
  int32_t max_chunk;         /* most prompt rows one request brings to one pass (>= 1); longer
                                prompts continue in the next pass (chunked prefill) */
  int32_t max_tokens;        /* most rows per pass; the workspace must cover this many tokens */
} ls_server_config;

/* What one pass did. */
typedef struct {
  int32_t n_batch;          /* requests in the batch after admission */
  int32_t n_new;            /* of these, admitted by this pass */
  int32_t n_decode;         /* decode rows executed */
  int32_t n_prefill;        /* prompt chunks executed */
  int32_t n_rows;           /* rows executed = n_decode + sum of chunk lengths; 0: nothing launched */
  int32_t n_stalled;        /* batch members left out of this pass (pages of the whole sequence cannot be
                               set aside yet, or the pass has no chunk or row left) */
  int32_t n_finished;       /* requests that completed with this pass */
  int32_t free_pages;       /* pages in no request's hands, after the pass */
  int32_t unreserved_pages; /* pages that no started request has set aside, after the pass: a waiting
                               request starts when its ceil((prompt_len + n_decode) / page_size) fit here */
} ls_pass_report;

/* k_pool, v_pool [dev]: as in ls_kv, with cfg->n_pages pages.  LS_EINVAL for
 * bad sizes, LS_ENOMEM when the server's buffers cannot be allocated. */
ls_status ls_server_create(ls_stage* s, const ls_server_config* cfg, void* k_pool, void* v_pool,
                           ls_server** out);
void ls_server_destroy(ls_server* sv);

/* Enqueues an inference request (FCFS).  id >= 0 and not in flight;
 * prompt_len >= 1, n_decode >= 0; prompt_len + n_decode must fit
 * max_pages_per_req pages and the stage's max_pos. */
ls_status ls_server_submit(ls_server* sv, int64_t id, const void* X, void* Y, int prompt_len, int n_decode);

/*
 * One pass of Algorithm 3's loop body at time `now`: admission, then one
 * stage_step over the decode rows and prompt chunks of the batch (decode rows
 * first, then the chunks, each group in batch order), then the filter of
 * finished requests.  workspace [dev]: ls_workspace_bytes(s, max_tokens).
 * batch_ids / finished_ids [host], capacity max_batch each, may be null:
 * the ids of the requests that ran in this pass (decode rows first) and of
 * those that finished.
 */
ls_status ls_server_pass(ls_server* sv, double now, void* workspace, void* stream, ls_pass_report* report,
                         int64_t* ran_ids, int64_t* finished_ids);

/* Requests waiting for admission plus requests in the batch. */
int ls_server_in_flight(const ls_server* sv);

#ifdef __cplusplus
}
#endif
#endif /* LEMIX_SERVE_H */
