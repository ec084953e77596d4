// Asynchronous automaton construction (paper Sec. 5.4.2, asynchronous SAM construction; Alg. 4 step 2).
//
// Building the automaton of a long prompt would sit on the time to first token, so it is handed to a
// child thread: a request's prompt and, later, its generated tokens are put into a waiting queue and
// the call returns at once; the child thread works through the queue; while a request still has
// entries waiting, its automaton is not available yet and the caller decodes that request without
// drafts.  One builder owns one child thread and the automata of all the requests submitted to it.
// Flattening a grown automaton again (when its overlay of new transitions is no longer small) goes
// through the same queue, so it too stays off the decoding thread and is ordered with the appends.
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <memory>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_map>
#include <vector>

#include "agentsam.h"

namespace {

struct Request {
    sam_t *sam = nullptr;
    int64_t pending_entries = 0;     // queue entries (and the one being processed) not yet in the automaton
    int64_t pending_tokens = 0;
    int error = AGENTSAM_OK;         // first error of a background append (e.g. a negative token id)
    int flatten_rc = AGENTSAM_ERR_ARG;   // result of the last background flatten (ERR_ARG: none yet)
    bool released = false;           // forget it as soon as nothing is pending
};

struct FlattenJob {                  // where a background flatten writes (the caller's host arrays) and how much fits
    int32_t state_base, edge_base, corpus_base;
    int32_t *len, *link, *row_ptr, *edge_tok, *edge_dst, *lastpos, *corpus, *state_rec;
    int64_t cap_states, cap_edges, cap_tokens;
};

struct Entry {
    int64_t id;
    std::vector<int32_t> tokens;
    int32_t sep;
    bool flatten = false;
    FlattenJob job{};
};

}  // namespace

struct sam_builder {
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::deque<Entry> queue;
    std::unordered_map<int64_t, Request> req;
    bool stop = false;
    std::thread worker;

    void run() {
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            cv_work.wait(lk, [&] { return stop || !queue.empty(); });
            if (queue.empty()) return;                       // stop requested and nothing left to do
            Entry e = std::move(queue.front());
            queue.pop_front();
            Request &r = req[e.id];
            sam_t *target = r.sam;
            const bool skip = r.error != AGENTSAM_OK || r.released;
            lk.unlock();
            // the automaton of a request with pending entries is touched by this thread only
            int rc = AGENTSAM_OK;
            if (!skip && e.flatten) {
                const FlattenJob &j = e.job;
                int64_t ns = 0, ne = 0, nt = 0;
                if (!target) rc = AGENTSAM_ERR_ARG;          // nothing was ever submitted for this request
                else {
                    sam_flat_sizes(target, &ns, &ne, &nt);
                    if (ns > j.cap_states || ne > j.cap_edges || nt > j.cap_tokens) rc = AGENTSAM_ERR_WORKSPACE;
                    else rc = sam_flatten(target, j.state_base, j.edge_base, j.corpus_base, j.len, j.link, j.row_ptr,
                                          j.edge_tok, j.edge_dst, j.lastpos, j.corpus, j.state_rec);
                }
            } else if (!skip) {
                if (!target) rc = sam_build(e.tokens.data(), (int64_t)e.tokens.size(), e.sep, &target);
                else rc = sam_append(target, e.tokens.data(), (int64_t)e.tokens.size());
            }
            lk.lock();
            Request &r2 = req[e.id];
            if (!skip && e.flatten) {
                r2.flatten_rc = rc;                          // (a flatten that does not fit leaves the automaton usable)
            } else if (!skip) {
                if (rc != AGENTSAM_OK) r2.error = rc;
                else r2.sam = target;
            }
            r2.pending_entries -= 1;
            r2.pending_tokens -= (int64_t)e.tokens.size();
            if (r2.released && r2.pending_entries == 0) {
                sam_free(r2.sam);
                req.erase(e.id);
            }
            cv_done.notify_all();
        }
    }
};

extern "C" {

int sam_builder_create(sam_builder_t **out) {
    if (!out) return AGENTSAM_ERR_NULL;
    *out = nullptr;
    sam_builder *b = new (std::nothrow) sam_builder();
    if (!b) return AGENTSAM_ERR_NOMEM;
    try {
        b->worker = std::thread([b] { b->run(); });
    } catch (...) {
        delete b;
        return AGENTSAM_ERR_NOMEM;
    }
    *out = b;
    return AGENTSAM_OK;
}

int sam_builder_submit(sam_builder_t *b, int64_t request_id, const int32_t *tokens, int64_t n, int32_t sep_token) {
    if (!b || (n > 0 && !tokens)) return AGENTSAM_ERR_NULL;
    if (n < 0) return AGENTSAM_ERR_ARG;
    try {
        Entry e{request_id, std::vector<int32_t>(tokens, tokens + n), sep_token};
        std::lock_guard<std::mutex> lk(b->mu);
        Request &r = b->req[request_id];
        if (r.released) return AGENTSAM_ERR_ARG;             // released and still draining
        r.pending_entries += 1;
        r.pending_tokens += n;
        b->queue.push_back(std::move(e));
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    b->cv_work.notify_one();
    return AGENTSAM_OK;
}

int sam_builder_flatten(sam_builder_t *b, int64_t request_id, int32_t state_base, int32_t edge_base, int32_t corpus_base,
                        int32_t *len, int32_t *link, int32_t *row_ptr, int32_t *edge_tok, int32_t *edge_dst,
                        int32_t *lastpos, int32_t *corpus, int32_t *state_rec, int64_t cap_states, int64_t cap_edges,
                        int64_t cap_tokens) {
    if (!b || !len || !link || !row_ptr || !edge_tok || !edge_dst || !lastpos || !corpus || !state_rec) return AGENTSAM_ERR_NULL;
    if (cap_states < 1 || cap_edges < 0 || cap_tokens < 0 || state_base < 0 || edge_base < 0 || corpus_base < 0) return AGENTSAM_ERR_ARG;
    try {
        Entry e{request_id, {}, 0, true,
                FlattenJob{state_base, edge_base, corpus_base, len, link, row_ptr, edge_tok, edge_dst, lastpos, corpus,
                           state_rec, cap_states, cap_edges, cap_tokens}};
        std::lock_guard<std::mutex> lk(b->mu);
        auto it = b->req.find(request_id);
        if (it == b->req.end() || it->second.released) return AGENTSAM_ERR_ARG;
        it->second.pending_entries += 1;
        b->queue.push_back(std::move(e));
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    b->cv_work.notify_one();
    return AGENTSAM_OK;
}

int sam_builder_flatten_result(sam_builder_t *b, int64_t request_id) {
    if (!b) return AGENTSAM_ERR_NULL;
    std::lock_guard<std::mutex> lk(b->mu);
    auto it = b->req.find(request_id);
    if (it == b->req.end() || it->second.released) return AGENTSAM_ERR_ARG;
    return it->second.flatten_rc;
}

int sam_builder_poll(sam_builder_t *b, int64_t request_id, sam_t **out, int64_t *pending_tokens) {
    if (!b || !out) return AGENTSAM_ERR_NULL;
    *out = nullptr;
    std::lock_guard<std::mutex> lk(b->mu);
    auto it = b->req.find(request_id);
    if (it == b->req.end() || it->second.released) return AGENTSAM_ERR_ARG;
    if (pending_tokens) *pending_tokens = it->second.pending_tokens;
    if (it->second.error != AGENTSAM_OK) return it->second.error;
    if (it->second.pending_entries == 0) *out = it->second.sam;
    return AGENTSAM_OK;
}

int sam_builder_wait(sam_builder_t *b, int64_t request_id) {
    if (!b) return AGENTSAM_ERR_NULL;
    std::unique_lock<std::mutex> lk(b->mu);
    auto it = b->req.find(request_id);
    if (it == b->req.end()) return AGENTSAM_ERR_ARG;
    b->cv_done.wait(lk, [&] {
        auto jt = b->req.find(request_id);
        return jt == b->req.end() || jt->second.pending_entries == 0;
    });
    auto jt = b->req.find(request_id);
    return jt == b->req.end() ? AGENTSAM_OK : jt->second.error;
}

int sam_builder_release(sam_builder_t *b, int64_t request_id) {
    if (!b) return AGENTSAM_ERR_NULL;
    std::lock_guard<std::mutex> lk(b->mu);
    auto it = b->req.find(request_id);
    if (it == b->req.end() || it->second.released) return AGENTSAM_ERR_ARG;
    if (it->second.pending_entries == 0) {
        sam_free(it->second.sam);
        b->req.erase(it);
    } else {
        it->second.released = true;                          // the child thread drops it when it gets there
    }
    return AGENTSAM_OK;
}

void sam_builder_destroy(sam_builder_t *b) {
    if (!b) return;
    {
        std::lock_guard<std::mutex> lk(b->mu);
        b->stop = true;
        b->queue.clear();                                    // whatever is still waiting is abandoned
    }
    b->cv_work.notify_all();
    if (b->worker.joinable()) b->worker.join();
    for (auto &kv : b->req) sam_free(kv.second.sam);
    delete b;
}

}  // extern "C"
