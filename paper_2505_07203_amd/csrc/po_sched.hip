// Host-side request scheduler: shortest-remaining-job-first with continuous JCT calibration
// (Section 6.3, Algorithm 1).  Every pick re-evaluates the job completion time of every waiting
// request against what the prefix cache holds NOW, so that requests that can hit the prefix a
// just-finished request left behind are taken before the cache moves on; the queuing time, scaled
// by lambda, is subtracted against starvation.  No device code: plain C++ behind the C ABI;
// po_engine_step joins the scheduler to a context through the library's own public calls.
#include "../../include/po.h"

#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <vector>

struct po_sched {
    double lambda;
    bool linear;              // false: the paper's default proxy n_input - n_cached
    double c0, c_input, c_cached;
    struct Req {
        int64_t id;
        double arrival;
        std::vector<int32_t> tokens;
        std::vector<int32_t> cand;      // the request's own acceptable output tokens (may be empty)
    };
    std::vector<Req> queue;   // push order
};

namespace {

int64_t hit_len(const std::vector<int32_t>& t, const int32_t* cached, int64_t n_cached_tokens) {
    // common prefix with the cache; one position of a request is always computed
    const int64_t lim = std::min<int64_t>((int64_t)t.size() - 1, n_cached_tokens);
    int64_t m = 0;
    while (m + 64 <= lim && memcmp(t.data() + m, cached + m, 64 * sizeof(int32_t)) == 0) m += 64;   // whole blocks first
    while (m < lim && t[(size_t)m] == cached[m]) ++m;
    return m;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

po_status po_sched_create(double lambda, po_sched** out) {
    if (!out || !(lambda >= 0.0)) return PO_ERR_INVALID_ARG;
    po_sched* s = new (std::nothrow) po_sched();
    if (!s) return PO_ERR_OOM;
    s->lambda = lambda;
    s->linear = false;
    s->c0 = s->c_input = s->c_cached = 0.0;
    *out = s;
    return PO_OK;
}

void po_sched_destroy(po_sched* s) { delete s; }

po_status po_sched_set_jct_model(po_sched* s, double c0, double c_input, double c_cached) {
    if (!s || !std::isfinite(c0) || !std::isfinite(c_input) || !std::isfinite(c_cached)) return PO_ERR_INVALID_ARG;
    s->linear = true;
    s->c0 = c0;
    s->c_input = c_input;
    s->c_cached = c_cached;
    return PO_OK;
}

po_status po_sched_fit_jct_model(po_sched* s, const int64_t* n_input, const int64_t* n_cached, const double* jct,
                                 int32_t n, double coef[3]) {
    if (!s || !n_input || !n_cached || !jct || n < 3) return PO_ERR_INVALID_ARG;
    // normal equations of jct ~ c0 + c_input * n_input + c_cached * n_cached, centred for conditioning
    double mx = 0, my = 0, mz = 0;
    for (int32_t i = 0; i < n; ++i) { mx += (double)n_input[i]; my += (double)n_cached[i]; mz += jct[i]; }
    mx /= n; my /= n; mz /= n;
    double sxx = 0, sxy = 0, syy = 0, sxz = 0, syz = 0;
    for (int32_t i = 0; i < n; ++i) {
        const double x = (double)n_input[i] - mx, y = (double)n_cached[i] - my, z = jct[i] - mz;
        sxx += x * x; sxy += x * y; syy += y * y; sxz += x * z; syz += y * z;
    }
    const double det = sxx * syy - sxy * sxy;
    if (!(std::fabs(det) > 1e-12 * (sxx * syy + 1e-300))) return PO_ERR_INVALID_ARG;    // collinear samples
    const double a = (sxz * syy - syz * sxy) / det, b = (syz * sxx - sxz * sxy) / det;
    s->linear = true;
    s->c_input = a;
    s->c_cached = b;
    s->c0 = mz - a * mx - b * my;
    if (coef) { coef[0] = s->c0; coef[1] = a; coef[2] = b; }
    return PO_OK;
}

po_status po_sched_push_request(po_sched* s, int64_t id, const int32_t* tokens, int64_t len, const int32_t* cand_ids,
                                int32_t n_cand, double arrival_time) {
    if (!s || !tokens || len <= 0 || !std::isfinite(arrival_time) || n_cand < 0 || (n_cand > 0 && !cand_ids))
        return PO_ERR_INVALID_ARG;
    po_sched::Req r;
    r.id = id;
    r.arrival = arrival_time;
    r.tokens.assign(tokens, tokens + len);
    if (n_cand > 0) r.cand.assign(cand_ids, cand_ids + n_cand);
    s->queue.push_back(std::move(r));
    return PO_OK;
}

po_status po_sched_push(po_sched* s, int64_t id, const int32_t* tokens, int64_t len, double arrival_time) {
    return po_sched_push_request(s, id, tokens, len, nullptr, 0, arrival_time);
}

int64_t po_sched_size(const po_sched* s) { return s ? (int64_t)s->queue.size() : 0; }

po_status po_sched_pick_multi(po_sched* s, const int32_t* const* cached_tokens, const int64_t* n_cached_tokens,
                              int32_t n_entries, double now, int64_t* id, int64_t* n_cached_hit) {
    if (!s || !id || n_entries < 0 || (n_entries > 0 && (!cached_tokens || !n_cached_tokens))) return PO_ERR_INVALID_ARG;
    for (int32_t e = 0; e < n_entries; ++e)
        if (n_cached_tokens[e] < 0 || (n_cached_tokens[e] > 0 && !cached_tokens[e])) return PO_ERR_INVALID_ARG;
    *id = -1;
    if (n_cached_hit) *n_cached_hit = 0;
    size_t best = 0;
    int64_t best_hit = 0;
    double best_score = std::numeric_limits<double>::infinity();
    bool found = false;
    for (size_t i = 0; i < s->queue.size(); ++i) {
        const po_sched::Req& r = s->queue[i];
        int64_t hit = 0;            // the best any cache entry offers this request
        for (int32_t e = 0; e < n_entries; ++e) hit = std::max(hit, hit_len(r.tokens, cached_tokens[e], n_cached_tokens[e]));
        const double n_in = (double)r.tokens.size();
        const double jct = s->linear ? s->c0 + s->c_input * n_in + s->c_cached * (double)hit : n_in - (double)hit;
        const double score = jct - s->lambda * (now - r.arrival);
        if (!found || score < best_score) { best = i; best_score = score; best_hit = hit; found = true; }
    }
    if (!found) return PO_OK;
    *id = s->queue[best].id;
    if (n_cached_hit) *n_cached_hit = best_hit;
    s->queue.erase(s->queue.begin() + (std::ptrdiff_t)best);
    return PO_OK;
}

po_status po_engine_step(po_ctx* ctx, po_sched* s, double now, const int32_t* cand_ids, int32_t n_cand,
                         float* out_logits, float* out_cand_logprobs, int32_t cand_capacity, int64_t* id, int64_t* len,
                         int64_t* reused_prefix_len, int32_t* n_cand_used) {
    if (!ctx || !s || !id || n_cand < 0 || cand_capacity < 0 || (cand_ids && n_cand == 0)) return PO_ERR_INVALID_ARG;
    *id = -1;
    if (n_cand_used) *n_cand_used = 0;
    if (len) *len = 0;
    if (reused_prefix_len) *reused_prefix_len = 0;
    if (s->queue.empty()) return PO_OK;
    int64_t n_slot0 = 0;
    const bool cached = po_kv_cache_slot(ctx, 0, nullptr, 0, &n_slot0) == PO_OK;      // a cache is attached
    size_t best = 0;
    double best_score = std::numeric_limits<double>::infinity();
    for (size_t i = 0; i < s->queue.size(); ++i) {
        const po_sched::Req& r = s->queue[i];
        int64_t hit = 0;
        if (cached) {
            const po_status st = po_kv_cache_match(ctx, r.tokens.data(), (int64_t)r.tokens.size(), &hit);
            if (st != PO_OK) return st;
        }
        const double n_in = (double)r.tokens.size();
        const double jct = s->linear ? s->c0 + s->c_input * n_in + s->c_cached * (double)hit : n_in - (double)hit;
        const double score = jct - s->lambda * (now - r.arrival);
        if (i == 0 || score < best_score) { best = i; best_score = score; }
    }
    // the acceptable-token list: the caller's for whichever request runs, else the request's own; the output
    // buffer must hold it (checked before the request leaves the queue)
    const bool own = cand_ids == nullptr;
    if (own) n_cand = (int32_t)s->queue[best].cand.size();
    if (out_cand_logprobs && n_cand > cand_capacity) return PO_ERR_INVALID_ARG;
    // The request leaves the queue only once it has run: one that the context refuses (too long for it, a token id
    // out of range) or whose run fails stays queued and is named in *id, so that the caller can drop it
    // (po_sched_remove) or try again; nothing is lost on an error.
    const po_sched::Req& r = s->queue[best];
    if (own) cand_ids = r.cand.empty() ? nullptr : r.cand.data();
    *id = r.id;
    if (len) *len = (int64_t)r.tokens.size();
    const po_status st =
        cached ? po_prefill_prefix(ctx, r.tokens.data(), (int64_t)r.tokens.size(), PO_KEEP_ALL, cand_ids, n_cand, out_logits,
                                   out_cand_logprobs, reused_prefix_len)
               : po_prefill(ctx, r.tokens.data(), (int64_t)r.tokens.size(), cand_ids, n_cand, out_logits, out_cand_logprobs);
    if (st != PO_OK) return st;
    if (n_cand_used) *n_cand_used = out_cand_logprobs ? n_cand : 0;
    s->queue.erase(s->queue.begin() + (std::ptrdiff_t)best);
    return PO_OK;
}

po_status po_sched_remove(po_sched* s, int64_t id) {
    if (!s) return PO_ERR_INVALID_ARG;
    for (size_t i = 0; i < s->queue.size(); ++i)
        if (s->queue[i].id == id) {
            s->queue.erase(s->queue.begin() + (std::ptrdiff_t)i);
            return PO_OK;
        }
    return PO_ERR_INVALID_ARG;
}

po_status po_sched_pick(po_sched* s, const int32_t* cached_tokens, int64_t n_cached_tokens, double now, int64_t* id,
                        int64_t* n_cached_hit) {
    if (n_cached_tokens < 0 || (n_cached_tokens > 0 && !cached_tokens)) return PO_ERR_INVALID_ARG;
    return po_sched_pick_multi(s, &cached_tokens, &n_cached_tokens, 1, now, id, n_cached_hit);
}

#pragma GCC visibility pop
}
