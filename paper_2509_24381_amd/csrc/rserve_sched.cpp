// Host side of include/rserve_sched.h: the per-request embedding tracker (section 3.1), encoder batching (Algorithm 1)
// and the schedulable-token scheduler (Algorithm 2).  Integer bookkeeping only; nothing here touches the GPU.
#include "../../include/rserve_sched.h"

#include <algorithm>
#include <deque>
#include <unordered_map>
#include <vector>

#include "last_error.h"

namespace {

// Tracker entry of one request: its segments with readiness tags, and the prefill cursor.
struct Request {
    int64_t id = 0;
    std::vector<rs_segment> segs;
    std::vector<char> ready;     // readiness tag per segment
    std::vector<int> seg_begin;  // first token of each segment
    int prompt_len = 0;
    int prefilled = 0;           // tokens already handed to a micro-batch
    int cursor_seg = 0;          // segment that holds token `prefilled` (== segs.size() when finished)

    // Length of the run of ready tokens that starts at the cursor.
    int schedulable() const {
        int end = prefilled;
        for (size_t i = cursor_seg; i < segs.size() && ready[i]; ++i) end = seg_begin[i] + segs[i].n_tokens;
        return end - prefilled;
    }
    void advance(int n) {
        prefilled += n;
        while (cursor_seg < (int)segs.size() && prefilled >= seg_begin[cursor_seg] + segs[cursor_seg].n_tokens) ++cursor_seg;
    }
    bool finished() const { return prefilled == prompt_len; }
};

}  // namespace

struct rs_sched {
    int budget = 0;
    std::unordered_map<int64_t, Request> tracker;  // request id -> entry (section 3.4: a dictionary keyed by request id)
    std::deque<int64_t> queue;                     // Q, head first
};

namespace {

const Request* find(const rs_sched* s, int64_t id) {
    if (!s) return nullptr;
    auto it = s->tracker.find(id);
    return it == s->tracker.end() ? nullptr : &it->second;
}

}  // namespace

extern "C" {

rs_status rs_sched_create(int token_budget, rs_sched** out) {
    if (!out) return rs_internal_fail(RS_EINVAL, "out is null");
    *out = nullptr;
    if (token_budget <= 0) return rs_internal_fail(RS_EINVAL, "token_budget = %d must be positive", token_budget);
    rs_sched* s = new rs_sched();
    s->budget = token_budget;
    *out = s;
    return RS_OK;
}

void rs_sched_destroy(rs_sched* s) { delete s; }

rs_status rs_sched_add_request(rs_sched* s, int64_t request_id, const rs_segment* segments, int n_segments) {
    if (!s || !segments) return rs_internal_fail(RS_EINVAL, "null argument");
    if (n_segments <= 0) return rs_internal_fail(RS_EINVAL, "n_segments = %d must be positive", n_segments);
    if (s->tracker.count(request_id)) return rs_internal_fail(RS_EINVAL, "request %lld already exists", (long long)request_id);
    Request r;
    r.id = request_id;
    long total = 0;
    for (int i = 0; i < n_segments; ++i) {
        if (segments[i].n_tokens <= 0) return rs_internal_fail(RS_EINVAL, "segment %d has %d tokens", i, segments[i].n_tokens);
        r.seg_begin.push_back((int)total);
        total += segments[i].n_tokens;
        if (total > 0x3fffffff) return rs_internal_fail(RS_EINVAL, "prompt too long");
        r.segs.push_back(segments[i]);
        r.ready.push_back(segments[i].is_mm ? 0 : 1);  // text embeddings exist from the start
    }
    r.prompt_len = (int)total;
    s->tracker.emplace(request_id, std::move(r));
    s->queue.push_back(request_id);
    return RS_OK;
}

rs_status rs_sched_mark_ready(rs_sched* s, int64_t request_id, int segment) {
    if (!s) return rs_internal_fail(RS_EINVAL, "scheduler is null");
    auto it = s->tracker.find(request_id);
    if (it == s->tracker.end()) return rs_internal_fail(RS_EINVAL, "unknown request %lld", (long long)request_id);
    Request& r = it->second;
    if (segment < 0 || segment >= (int)r.segs.size()) return rs_internal_fail(RS_EINVAL, "segment %d out of range", segment);
    if (!r.segs[segment].is_mm) return rs_internal_fail(RS_EINVAL, "segment %d is text", segment);
    r.ready[segment] = 1;
    return RS_OK;
}

int rs_sched_schedulable_tokens(const rs_sched* s, int64_t request_id) {
    const Request* r = find(s, request_id);
    return r ? r->schedulable() : -1;
}

int rs_sched_prompt_length(const rs_sched* s, int64_t request_id) {
    const Request* r = find(s, request_id);
    return r ? r->prompt_len : -1;
}

int rs_sched_prefilled_tokens(const rs_sched* s, int64_t request_id) {
    const Request* r = find(s, request_id);
    return r ? r->prefilled : -1;
}

rs_status rs_sched_encoder_batches(const rs_sched* s, int64_t request_id, int min_tokens, rs_encode_batch* out, int capacity,
                                   int* n_batches) {
    if (!s || !n_batches) return rs_internal_fail(RS_EINVAL, "null argument");
    *n_batches = 0;
    const Request* r = find(s, request_id);
    if (!r) return rs_internal_fail(RS_EINVAL, "unknown request %lld", (long long)request_id);
    if (min_tokens <= 0) return rs_internal_fail(RS_EINVAL, "min_tokens = %d must be positive", min_tokens);
    if (capacity < 0 || (capacity > 0 && !out)) return rs_internal_fail(RS_EINVAL, "bad output array");
    std::vector<rs_encode_batch> batches;
    rs_encode_batch buf{-1, -1, 0, 0};
    for (int i = 0; i < (int)r->segs.size(); ++i) {
        if (!r->segs[i].is_mm) continue;
        if (buf.n_items == 0) buf.first_segment = i;
        buf.last_segment = i;
        buf.n_items += 1;
        buf.n_tokens += r->segs[i].n_tokens;
        if (buf.n_tokens >= min_tokens) {  // Encode(buffer); buffer <- empty
            batches.push_back(buf);
            buf = rs_encode_batch{-1, -1, 0, 0};
        }
    }
    if (buf.n_items > 0) batches.push_back(buf);  // remaining multimodal data
    if ((int)batches.size() > capacity)
        return rs_internal_fail(RS_EWORKSPACE, "%zu batches do not fit capacity %d", batches.size(), capacity);
    std::copy(batches.begin(), batches.end(), out);
    *n_batches = (int)batches.size();
    return RS_OK;
}

rs_status rs_sched_next_round(rs_sched* s, rs_round_entry* entries, int capacity, int* n_entries) {
    if (!s || !n_entries) return rs_internal_fail(RS_EINVAL, "null argument");
    *n_entries = 0;
    if (capacity < 0 || (capacity > 0 && !entries)) return rs_internal_fail(RS_EINVAL, "bad output array");
    // decide the round first (no state change if the output does not fit)
    std::vector<rs_round_entry> S;
    int B = s->budget;
    size_t visited = 0;
    while (visited < s->queue.size() && B > 0) {
        const Request& r = s->tracker.at(s->queue[visited]);
        ++visited;
        const int t = r.schedulable();
        const int n = std::min(t, B);  // t <= B: all of them; t > B: what the budget still allows
        B -= n;
        S.push_back(rs_round_entry{r.id, r.prefilled, n, r.prefilled + n == r.prompt_len ? 1 : 0});
    }
    if ((int)S.size() > capacity) return rs_internal_fail(RS_EWORKSPACE, "%zu entries do not fit capacity %d", S.size(), capacity);
    // commit: advance cursors; unfinished visited requests (U) return to the head of Q in their order, finished ones leave
    std::deque<int64_t> U;
    for (const rs_round_entry& e : S) {
        Request& r = s->tracker.at(e.request_id);
        r.advance(e.n_tokens);
        if (!r.finished()) U.push_back(r.id);
    }
    s->queue.erase(s->queue.begin(), s->queue.begin() + (long)visited);
    s->queue.insert(s->queue.begin(), U.begin(), U.end());
    std::copy(S.begin(), S.end(), entries);
    *n_entries = (int)S.size();
    return RS_OK;
}

int rs_sched_queue_length(const rs_sched* s) { return s ? (int)s->queue.size() : -1; }

rs_status rs_sched_queue_ids(const rs_sched* s, int64_t* ids, int capacity, int* n_ids) {
    if (!s || !n_ids) return rs_internal_fail(RS_EINVAL, "null argument");
    *n_ids = 0;
    if (capacity < 0 || (capacity > 0 && !ids)) return rs_internal_fail(RS_EINVAL, "bad output array");
    const int n = std::min<int>(capacity, (int)s->queue.size());
    std::copy(s->queue.begin(), s->queue.begin() + n, ids);
    *n_ids = n;
    return RS_OK;
}

rs_status rs_sched_release_request(rs_sched* s, int64_t request_id) {
    if (!s) return rs_internal_fail(RS_EINVAL, "scheduler is null");
    auto it = s->tracker.find(request_id);
    if (it == s->tracker.end()) return rs_internal_fail(RS_EINVAL, "unknown request %lld", (long long)request_id);
    s->tracker.erase(it);
    s->queue.erase(std::remove(s->queue.begin(), s->queue.end(), request_id), s->queue.end());
    return RS_OK;
}

}  // extern "C"
