// Multi-step Pilot-Commit scheduling (Algorithm 1; Section 3.4: replay buffer, maximum delay, eviction).
// Host-side bookkeeping only: no device code, no HIP calls.
#include <deque>
#include <new>
#include <unordered_set>
#include <vector>

#include "pc_internal.h"

struct pc_sched {
    struct Entry {
        int64_t uid, tag;
        int64_t t0;   // step of the pilot pass that kept the prompt
    };
    pc_sched_config cfg;
    int64_t t = 0;
    int rounds_this_step = 0;
    std::deque<Entry> buffer;   // insertion order: step stamps never decrease
    std::unordered_set<int64_t> evicted;
    int64_t stats[PC_SCHED_NSTATS] = {0};
};

using pc::set_error;

extern "C" {

pc_status pc_sched_create(const pc_sched_config *cfg, pc_sched **out) {
    if (!cfg || !out) {
        set_error("pc_sched_create: null argument");
        return PC_ERR_INVALID_ARG;
    }
    if (cfg->b_t <= 0 || cfg->max_delay < 0 || !(cfg->p_lower <= cfg->p_upper)) {
        set_error("pc_sched_create: need b_t > 0, max_delay >= 0, p_lower <= p_upper (got %d, %d, %g, %g)", cfg->b_t,
                  cfg->max_delay, cfg->p_lower, cfg->p_upper);
        return PC_ERR_INVALID_ARG;
    }
    pc_sched *s = new (std::nothrow) pc_sched;
    if (!s) {
        set_error("pc_sched_create: out of host memory");
        return PC_ERR_OOM;
    }
    s->cfg = *cfg;
    *out = s;
    return PC_OK;
}

pc_status pc_sched_destroy(pc_sched *s) {
    delete s;
    return PC_OK;
}

pc_status pc_sched_pilot(pc_sched *s, const int64_t *prompt_uid, const int64_t *tag, const float *p_hat, int32_t n,
                         uint8_t *cls, uint8_t *evict, int32_t *counts) {
    if (!s || n < 0 || (n > 0 && (!prompt_uid || !p_hat))) {
        set_error("pc_sched_pilot: null argument or negative n");
        return PC_ERR_INVALID_ARG;
    }
    int32_t kept = 0, ev = 0, easy = 0, hard = 0;
    const float lo = s->cfg.p_lower, hi = s->cfg.p_upper, solve = s->cfg.p_solve;
    // Growing the containers can run out of host memory.  Nothing may leave through the C boundary as an
    // exception, and a failed call leaves the state as it was: what was appended is taken back.
    const size_t buffer_before = s->buffer.size();
    std::vector<int64_t> newly_evicted;
    try {
        for (int32_t q = 0; q < n; ++q) {
            const float p = p_hat[q];
            if (p >= lo && p <= hi) s->buffer.push_back({prompt_uid[q], tag ? tag[q] : 0, s->t});
            if (p >= solve && s->evicted.insert(prompt_uid[q]).second) newly_evicted.push_back(prompt_uid[q]);
        }
    } catch (...) {
        s->buffer.resize(buffer_before);
        for (int64_t u : newly_evicted) s->evicted.erase(u);
        set_error("pc_sched_pilot: out of host memory");
        return PC_ERR_OOM;
    }
    for (int32_t q = 0; q < n; ++q) {
        const float p = p_hat[q];
        uint8_t c;
        if (p > hi) {
            c = 2;
            ++easy;
        } else if (p < lo) {
            c = 0;
            ++hard;
        } else {
            c = 1;
            ++kept;
        }
        const bool e = p >= solve;
        ev += e;
        if (cls) cls[q] = c;
        if (evict) evict[q] = e ? 1 : 0;
    }
    if (counts) {
        counts[0] = kept;
        counts[1] = ev;
        counts[2] = easy;
        counts[3] = hard;
    }
    ++s->rounds_this_step;
    s->stats[PC_SCHED_PILOT_BATCHES] += 1;
    s->stats[PC_SCHED_PROMPTS_SEEN] += n;
    s->stats[PC_SCHED_BUFFERED] += kept;
    s->stats[PC_SCHED_EVICTIONS] += ev;
    return PC_OK;
}

pc_status pc_sched_commit(pc_sched *s, int64_t *uid_out, int64_t *tag_out, int32_t *age_out, int32_t *n_selected,
                          int64_t *aged_uid_out, int64_t *aged_tag_out, int32_t aged_cap, int32_t *n_aged) {
    if (!s || !uid_out || !n_selected || aged_cap < 0) {
        set_error("pc_sched_commit: null argument or negative aged_cap");
        return PC_ERR_INVALID_ARG;
    }
    const int64_t t = s->t;
    const size_t nb = s->buffer.size();
    // the survivors of step t are the tail of the buffer (stamps never decrease)
    size_t first_cur = nb;
    while (first_cur > 0 && s->buffer[first_cur - 1].t0 == t) --first_cur;
    const size_t b_t = (size_t)s->cfg.b_t;
    const size_t n_cur = std::min(nb - first_cur, b_t);          // taken from the current step, in batch order
    const size_t n_old = std::min(first_cur, b_t - n_cur);       // then from the front: oldest first
    // what stays: [n_old, first_cur) and [first_cur + n_cur, nb); of those, the ones too old for step t+1 go
    size_t aged = 0;
    auto too_old = [&](const pc_sched::Entry &e) { return t + 1 - e.t0 > (int64_t)s->cfg.max_delay; };
    for (size_t i = n_old; i < first_cur; ++i) aged += too_old(s->buffer[i]);
    for (size_t i = first_cur + n_cur; i < nb; ++i) aged += too_old(s->buffer[i]);
    if ((aged_uid_out || aged_tag_out) && aged > (size_t)aged_cap) {
        set_error("pc_sched_commit: %zu entries age out, aged_cap is %d", aged, aged_cap);
        return PC_ERR_INVALID_ARG;
    }
    // the entries that stay, built first: this is the only step that can run out of memory, and nothing has
    // been written or changed yet
    std::deque<pc_sched::Entry> rest;
    try {
        for (size_t i = n_old; i < first_cur; ++i)
            if (!too_old(s->buffer[i])) rest.push_back(s->buffer[i]);
        for (size_t i = first_cur + n_cur; i < nb; ++i)
            if (!too_old(s->buffer[i])) rest.push_back(s->buffer[i]);
    } catch (...) {
        set_error("pc_sched_commit: out of host memory");
        return PC_ERR_OOM;
    }
    size_t k = 0;
    auto emit = [&](const pc_sched::Entry &e) {
        uid_out[k] = e.uid;
        if (tag_out) tag_out[k] = e.tag;
        if (age_out) age_out[k] = (int32_t)(t - e.t0);
        ++k;
    };
    for (size_t i = 0; i < n_cur; ++i) emit(s->buffer[first_cur + i]);
    for (size_t i = 0; i < n_old; ++i) emit(s->buffer[i]);
    size_t a = 0;
    auto report_aged = [&](const pc_sched::Entry &e) {
        if (!too_old(e)) return;
        if (aged_uid_out) aged_uid_out[a] = e.uid;
        if (aged_tag_out) aged_tag_out[a] = e.tag;
        ++a;
    };
    for (size_t i = n_old; i < first_cur; ++i) report_aged(s->buffer[i]);
    for (size_t i = first_cur + n_cur; i < nb; ++i) report_aged(s->buffer[i]);
    s->buffer.swap(rest);
    *n_selected = (int32_t)k;
    if (n_aged) *n_aged = (int32_t)a;
    s->stats[PC_SCHED_COMMITTED] += (int64_t)k;
    s->stats[PC_SCHED_AGED_OUT] += (int64_t)a;
    s->stats[PC_SCHED_SHORT_STEPS] += k < b_t;
    s->stats[PC_SCHED_MULTI_ROUND_STEPS] += s->rounds_this_step > 1;
    s->rounds_this_step = 0;
    s->t = t + 1;
    return PC_OK;
}

pc_status pc_sched_evicted(const pc_sched *s, const int64_t *prompt_uid, int32_t n, uint8_t *out) {
    if (!s || n < 0 || (n > 0 && (!prompt_uid || !out))) {
        set_error("pc_sched_evicted: null argument or negative n");
        return PC_ERR_INVALID_ARG;
    }
    for (int32_t i = 0; i < n; ++i) out[i] = s->evicted.count(prompt_uid[i]) ? 1 : 0;
    return PC_OK;
}

pc_status pc_sched_stats(const pc_sched *s, int64_t *out) {
    if (!s || !out) {
        set_error("pc_sched_stats: null argument");
        return PC_ERR_INVALID_ARG;
    }
    for (int i = 0; i < PC_SCHED_NSTATS; ++i) out[i] = s->stats[i];
    out[PC_SCHED_STEP] = s->t;
    out[PC_SCHED_BUFFERED_NOW] = (int64_t)s->buffer.size();
    return PC_OK;
}

}  // extern "C"
