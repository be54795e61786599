/*
 * rserve_sched.h -- C ABI of the host-side request bookkeeping that feeds rs_prefill_batch: RServe's per-request
 * embedding tracker (arXiv 2509.24381, section 3.1), its encoder batching (Algorithm 1, section 3.2) and its
 * schedulable-token scheduler (Algorithm 2, section 3.3).
 *
 * Everything here is integer bookkeeping on the host: no call touches the GPU, allocates device memory or needs a
 * device to be present.  A scheduling round returns, per request, which rows of the request's prompt go into the next
 * micro-batch; the caller gathers those embedding rows into the packed [sum T, H] input of rs_prefill_batch (one
 * rs_kv per request, chunk_lens = the rounds' n_tokens) and runs the layers.
 *
 * Model of a request (section 3.1).  A prompt is a sequence of segments, each either text (its embeddings exist when
 * the request is created: readiness tag true) or one multimodal item (an indivisible unit of the encoder; its tag is
 * false until rs_sched_mark_ready reports that the encoder has delivered its embeddings).  Tokens are prefilled
 * strictly in prompt order.  A token is schedulable when its embedding is ready and every token before it has been
 * prefilled or is schedulable too, so the number of schedulable tokens of a request is the length of the run of ready
 * tokens that starts at its prefill cursor.
 *
 * Readings of Algorithm 2 where the listing is loose (both stated in the functions' comments as well):
 *  - a request whose schedulable tokens t exceed the remaining budget B contributes B tokens (the listing adds it to S
 *    and sets B to 0 without saying how many of its tokens run);
 *  - "t < p" (mark as incomplete) is read as "the request still has tokens that are not prefilled after this round":
 *    as printed it compares the schedulable tokens of one round with the whole prompt length.
 *
 * Errors: RS_EINVAL for null pointers, unknown or duplicate ids, bad indices or sizes; RS_EWORKSPACE when an output
 * array is too small (nothing changes in that case).  Not thread-safe: one scheduler, one caller thread.
 */
#ifndef RSERVE_SCHED_H
#define RSERVE_SCHED_H

#include <stdint.h>

#include "rserve_prefill.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rs_sched rs_sched;

/* One element of a prompt: a run of text tokens, or one multimodal item of n_tokens embedding rows. */
typedef struct rs_segment {
    int is_mm;     /* 0: text, non-zero: multimodal item */
    int n_tokens;  /* > 0 */
} rs_segment;

/* One member of the micro-batch S of a scheduling round: rows [first_token, first_token + n_tokens) of the request's
 * prompt.  n_tokens may be 0 (the request was visited but is waiting for its encoder).  finished is non-zero when the
 * request's whole prompt is prefilled once this round has run. */
typedef struct rs_round_entry {
    int64_t request_id;
    int first_token;
    int n_tokens;
    int finished;
} rs_round_entry;

/* One Encode(buffer) call of Algorithm 1: the multimodal items among segments [first_segment, last_segment]. */
typedef struct rs_encode_batch {
    int first_segment;
    int last_segment;  /* inclusive; both ends are multimodal segments */
    int n_items;
    int n_tokens;
} rs_encode_batch;

/* token_budget: B of Algorithm 2, the most tokens one round may schedule (> 0). */
rs_status rs_sched_create(int token_budget, rs_sched** out);
void rs_sched_destroy(rs_sched* s);

/* Section 3.1: creates the request's tracker entry (text segments ready, multimodal segments not) and appends the
 * request to the tail of the waiting queue Q.  The segment array is copied. */
rs_status rs_sched_add_request(rs_sched* s, int64_t request_id, const rs_segment* segments, int n_segments);

/* Section 3.1: the encoder has produced the embeddings of multimodal segment `segment`; its readiness tag becomes
 * true.  Marking a ready segment again is a no-op; a text segment or an index out of range is RS_EINVAL. */
rs_status rs_sched_mark_ready(rs_sched* s, int64_t request_id, int segment);

/* SchedulableTokens(r), PromptLength(r) and the prefill cursor of a request; -1 for an unknown id. */
int rs_sched_schedulable_tokens(const rs_sched* s, int64_t request_id);
int rs_sched_prompt_length(const rs_sched* s, int64_t request_id);
int rs_sched_prefilled_tokens(const rs_sched* s, int64_t request_id);

/* Algorithm 1 for one request: walks its elements in order, buffers multimodal items, and closes a batch as soon as
 * the buffered items hold at least min_tokens (C) embedding rows; what remains at the end is a last, smaller batch.
 * Items are never split.  Writes at most capacity batches; *n_batches receives the count. */
rs_status rs_sched_encoder_batches(const rs_sched* s, int64_t request_id, int min_tokens, rs_encode_batch* out,
                                   int capacity, int* n_batches);

/* Algorithm 2, one iteration: dequeues requests from the head of Q while budget remains, gives each min(t, B) of its
 * schedulable tokens, advances the prefill cursors, drops finished requests from Q and puts the visited unfinished
 * ones back at the head in their original order.  entries (capacity >= rs_sched_queue_length) receives S in visiting
 * order, zero-token members included; *n_entries its size. */
rs_status rs_sched_next_round(rs_sched* s, rs_round_entry* entries, int capacity, int* n_entries);

/* Number of requests in Q (unfinished requests), and the queue's ids from head to tail (at most capacity of them). */
int rs_sched_queue_length(const rs_sched* s);
rs_status rs_sched_queue_ids(const rs_sched* s, int64_t* ids, int capacity, int* n_ids);

/* Forgets a request (finished or not): its tracker entry is released and it leaves Q. */
rs_status rs_sched_release_request(rs_sched* s, int64_t request_id);

#ifdef __cplusplus
}
#endif
#endif /* RSERVE_SCHED_H */
