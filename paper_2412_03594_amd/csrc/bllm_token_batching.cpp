// Throughput-oriented token batching on the host (BatchLLM Sec. 3.3): a job of prefix-sharing
// groups is played through iteration by iteration.  Groups take their turn in the order of
// R_group = 1 / (L_prefix + sum L_distinct), larger first (Eq. 3); every iteration fetches
// decode tokens, then distinct-prompt chunks, then common-prefix chunks (Sec. 3.3.1), bounded
// by the tokens per batch S_chunk and by the KV memory M_threshold instead of a request
// count (Sec. 3.3.3).  Each batch comes out in the form bllm_prefix_group_create_ex takes.
#include "bllm_internal.h"

#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

struct bllm_job {
    bllm_batching_params params;
    std::vector<int32_t> prefix_len, req_group, distinct, decode;
    std::vector<std::vector<int32_t>> members;
    std::vector<int32_t> prefix_queue, prompt_queue, decode_queue;     // in fetch order
    std::vector<int32_t> done_prefix, done_prompt, done_decode, unfinished;
    int64_t left = 0;        // unfinished requests
    int64_t kv = 0;          // KV tokens in use
    int32_t iteration = 0;
    // the batch handed out last (the view points into these)
    std::vector<int32_t> b_groups, b_prefix_len, b_prefix_q_len, b_requests, b_req_group, b_req_suffix_len, b_req_q_len;
    // per-iteration scratch
    std::vector<int32_t> rows_req, rows_prefix, group_slot;
};

using namespace bllm;

extern "C" int bllm_job_create(const bllm_batching_params* params, int32_t n_groups, const int32_t* prefix_len,
                               int32_t n_requests, const int32_t* req_group, const int32_t* req_distinct_len,
                               const int32_t* req_decode_len, bllm_job** out) {
    if (!params || !out || n_groups < 1 || n_requests < 0 || !prefix_len ||
        (n_requests > 0 && (!req_group || !req_distinct_len || !req_decode_len))) {
        set_error("null pointer argument, n_groups < 1 or n_requests < 0");
        return BLLM_INVALID_ARG;
    }
    if (params->s_chunk < 1 || params->m_threshold < 1 || params->max_requests < 0) {
        set_error("need s_chunk >= 1, m_threshold >= 1, max_requests >= 0");
        return BLLM_INVALID_ARG;
    }
    for (int32_t g = 0; g < n_groups; ++g)
        if (prefix_len[g] < 0) {
            set_error("negative prefix length in group " + std::to_string(g));
            return BLLM_INVALID_ARG;
        }
    for (int32_t r = 0; r < n_requests; ++r) {
        if (req_group[r] < 0 || req_group[r] >= n_groups) {
            set_error("request " + std::to_string(r) + ": group id out of range");
            return BLLM_INVALID_ARG;
        }
        if (req_distinct_len[r] < 0 || req_decode_len[r] < 1 || prefix_len[req_group[r]] + static_cast<int64_t>(req_distinct_len[r]) < 1) {
            set_error("request " + std::to_string(r) + ": need distinct_len >= 0, decode_len >= 1 and at least one prompt token");
            return BLLM_INVALID_ARG;
        }
        if (static_cast<int64_t>(req_distinct_len[r]) + req_decode_len[r] > INT32_MAX) {
            set_error("request " + std::to_string(r) + ": suffix length overflows int32");
            return BLLM_INVALID_ARG;
        }
    }
    try {
        bllm_job* j = new bllm_job();
        j->params = *params;
        j->prefix_len.assign(prefix_len, prefix_len + n_groups);
        j->req_group.assign(req_group, req_group + n_requests);
        j->distinct.assign(req_distinct_len, req_distinct_len + n_requests);
        j->decode.assign(req_decode_len, req_decode_len + n_requests);
        j->members.resize(n_groups);
        for (int32_t r = 0; r < n_requests; ++r) j->members[req_group[r]].push_back(r);
        // turn order of the groups: fewer prefill tokens (larger R_group) first, ties by index
        std::vector<int64_t> total(prefix_len, prefix_len + n_groups);
        for (int32_t r = 0; r < n_requests; ++r) total[req_group[r]] += req_distinct_len[r];
        std::vector<int32_t> order(n_groups);
        std::iota(order.begin(), order.end(), 0);
        if (params->reorder)
            std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return total[a] < total[b]; });
        for (int32_t g : order)
            if (!j->members[g].empty()) j->prefix_queue.push_back(g);
        j->done_prefix.assign(n_groups, 0);
        j->done_prompt.assign(n_requests, 0);
        j->done_decode.assign(n_requests, 0);
        j->unfinished.resize(n_groups);
        for (int32_t g = 0; g < n_groups; ++g) j->unfinished[g] = static_cast<int32_t>(j->members[g].size());
        j->left = n_requests;
        j->rows_req.assign(n_requests, 0);
        j->rows_prefix.assign(n_groups, 0);
        j->group_slot.assign(n_groups, -1);
        *out = j;
    } catch (const std::bad_alloc&) {
        set_error("out of host memory");
        return BLLM_OUT_OF_MEMORY;
    }
    return BLLM_OK;
}

extern "C" int bllm_job_next_batch(bllm_job* j, bllm_token_batch* out, int32_t* done) {
    if (!j || !out || !done) {
        set_error("null job, batch or done pointer");
        return BLLM_INVALID_ARG;
    }
    *out = bllm_token_batch{};
    if (j->left == 0) {
        *done = 1;
        return BLLM_OK;
    }
    *done = 0;
    const int64_t m = j->params.m_threshold;
    int64_t budget = j->params.s_chunk;
    int32_t seqs = 0;
    auto capped = [&] { return j->params.max_requests > 0 && seqs >= j->params.max_requests; };
    auto release_turn = [&](size_t at, bool only_with_distinct) {
        const int32_t g = j->prefix_queue[at];
        j->prefix_queue.erase(j->prefix_queue.begin() + static_cast<std::ptrdiff_t>(at));
        for (int32_t r : j->members[g])
            if (!only_with_distinct || j->distinct[r] > 0) j->prompt_queue.push_back(r);
    };
    std::vector<int32_t> sched_req, sched_groups;          // in fetch order
    // groups that share nothing and are at the head of the common-prefix queue: nothing to process first
    while (!j->prefix_queue.empty() && j->prefix_len[j->prefix_queue[0]] == 0) release_turn(0, false);
    int32_t n_dec = 0, n_dis = 0, n_pre = 0;
    // 1. decoding queue
    for (int32_t r : j->decode_queue) {
        if (budget == 0 || capped()) break;
        j->rows_req[r] = 1;
        sched_req.push_back(r);
        --budget;
        ++seqs;
        ++j->kv;
        ++n_dec;
    }
    // 2. distinct-prompt queue
    bool memory_full = false;
    for (int32_t r : j->prompt_queue) {
        if (budget == 0 || capped()) break;
        const int64_t chunk = std::min<int64_t>({j->distinct[r] - j->done_prompt[r], budget, m - j->kv});
        if (chunk <= 0) {
            memory_full = true;
            break;
        }
        j->rows_req[r] = static_cast<int32_t>(chunk);
        sched_req.push_back(r);
        budget -= chunk;
        ++seqs;
        j->kv += chunk;
        n_dis += static_cast<int32_t>(chunk);
    }
    // 3. common-prefix queue; the groups before `turn` have their whole prefix fetched
    size_t turn = 0;
    while (!memory_full && turn < j->prefix_queue.size()) {
        const int32_t g = j->prefix_queue[turn];
        if (j->prefix_len[g] == 0) {
            release_turn(turn, false);
            continue;
        }
        if (budget == 0 || capped()) break;
        const int64_t remaining = j->prefix_len[g] - j->done_prefix[g];
        const int64_t chunk = std::min<int64_t>({remaining, budget, m - j->kv});
        if (chunk <= 0) break;
        j->rows_prefix[g] = static_cast<int32_t>(chunk);
        sched_groups.push_back(g);
        budget -= chunk;
        ++seqs;
        j->kv += chunk;
        n_pre += static_cast<int32_t>(chunk);
        if (chunk < remaining) break;
        release_turn(turn, true);
    }
    if (sched_req.empty() && sched_groups.empty()) {
        set_error("no progress: m_threshold is too small for this job");
        return BLLM_UNSUPPORTED;
    }

    // ---- the batch, groups and requests ascending ----------------------------------------
    for (int32_t g : sched_groups) j->done_prefix[g] += j->rows_prefix[g];
    for (int32_t r : sched_req) {
        if (j->done_prompt[r] < j->distinct[r]) j->done_prompt[r] += j->rows_req[r];
        else j->done_decode[r] += j->rows_req[r];
    }
    j->b_groups = sched_groups;
    for (int32_t r : sched_req) j->b_groups.push_back(j->req_group[r]);
    std::sort(j->b_groups.begin(), j->b_groups.end());
    j->b_groups.erase(std::unique(j->b_groups.begin(), j->b_groups.end()), j->b_groups.end());
    j->b_prefix_len.clear();
    j->b_prefix_q_len.clear();
    for (size_t i = 0; i < j->b_groups.size(); ++i) {
        const int32_t g = j->b_groups[i];
        j->group_slot[g] = static_cast<int32_t>(i);
        j->b_prefix_len.push_back(j->done_prefix[g]);
        j->b_prefix_q_len.push_back(j->rows_prefix[g]);
    }
    j->b_requests = sched_req;
    std::sort(j->b_requests.begin(), j->b_requests.end());
    j->b_req_group.clear();
    j->b_req_suffix_len.clear();
    j->b_req_q_len.clear();
    for (int32_t r : j->b_requests) {
        j->b_req_group.push_back(j->group_slot[j->req_group[r]]);
        j->b_req_suffix_len.push_back(j->done_prompt[r] + j->done_decode[r]);
        j->b_req_q_len.push_back(j->rows_req[r]);
    }
    out->iteration = j->iteration++;
    out->n_groups = static_cast<int32_t>(j->b_groups.size());
    out->groups = j->b_groups.data();
    out->prefix_len = j->b_prefix_len.data();
    out->prefix_q_len = j->b_prefix_q_len.data();
    out->n_requests = static_cast<int32_t>(j->b_requests.size());
    out->requests = j->b_requests.data();
    out->req_group = j->b_req_group.data();
    out->req_suffix_len = j->b_req_suffix_len.data();
    out->req_q_len = j->b_req_q_len.data();
    out->n_decode_tokens = n_dec;
    out->n_distinct_tokens = n_dis;
    out->n_prefix_tokens = n_pre;
    out->kv_in_use = j->kv;

    // ---- end of the iteration: queue moves and releases ------------------------------------
    std::vector<int32_t> finished;
    auto prompt_complete = [&](int32_t r) {
        if (j->decode[r] >= 2) j->decode_queue.push_back(r);
        else finished.push_back(r);
    };
    {
        size_t keep = 0;
        const size_t n = j->decode_queue.size();
        for (size_t i = 0; i < n; ++i) {
            const int32_t r = j->decode_queue[i];
            if (j->rows_req[r] > 0 && j->done_decode[r] == j->decode[r] - 1) finished.push_back(r);
            else j->decode_queue[keep++] = r;
        }
        j->decode_queue.resize(keep);
    }
    {
        // requests that complete their prompt now join the decoding queue behind those already there
        std::vector<int32_t> still;
        for (int32_t r : j->prompt_queue) {
            if (j->rows_req[r] > 0 && j->done_prompt[r] == j->distinct[r]) prompt_complete(r);
            else still.push_back(r);
        }
        j->prompt_queue.swap(still);
    }
    for (int32_t g : sched_groups)
        if (j->done_prefix[g] == j->prefix_len[g])
            for (int32_t r : j->members[g])
                if (j->distinct[r] == 0) prompt_complete(r);
    for (int32_t r : finished) {
        j->kv -= j->done_prompt[r] + j->done_decode[r];
        const int32_t g = j->req_group[r];
        --j->left;
        if (--j->unfinished[g] == 0) j->kv -= j->prefix_len[g];
    }
    for (int32_t r : sched_req) j->rows_req[r] = 0;
    for (int32_t g : sched_groups) j->rows_prefix[g] = 0;
    return BLLM_OK;
}

extern "C" int bllm_job_destroy(bllm_job* j) {
    delete j;
    return BLLM_OK;
}
