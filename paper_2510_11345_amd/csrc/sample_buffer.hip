// SampleBuffer with the per-sample freshness rule of the asynchronous ratio (host only).
//
// ROLL Flash (arXiv 2510.11345) Section 4.3: the asynchronous ratio alpha is the largest allowed
// gap between the current policy version n and the version that initiated a sample; the buffer
// never holds a sample initiated before n - alpha, holds at most (1 + alpha) * batch samples, and
// no sample is wasted because none is started that would break the rule.  Section 4.2: ABORT
// interrupts a running request and reclaims it into the buffer for later recomputation, so a
// response may carry tokens of several policy versions while keeping its initiating version.
//
// Reading (the paper states the invariants, not the mechanism): a sample is *outstanding* from
// begin() until a batch takes it; one batch is taken per policy version.  A sample begun now,
// with k samples outstanding ahead of it, is consumed no earlier than floor(k / batch) batches
// from the next one, and the next batch belongs to this version only if it has not been taken
// yet; begin() is refused when that earliest version is already more than alpha ahead.  (So at
// most (1 + alpha) * batch samples are ever outstanding, and with alpha = 0 nothing starts while
// the trainer runs: the synchronous pipeline.)  take_batch() succeeds only if `batch` samples
// are complete and every sample that is due (it cannot wait for the next version) is complete;
// it takes the due ones first, then the oldest.  advance_version() is refused while a sample
// would become too old.  With these rules the capacity bound, the freshness bound and "nothing
// is dropped" hold for every interleaving (property-tested, also with ABORT / resume).
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "common.h"

struct roll_sample_buffer {
    int32_t batch = 0;
    double alpha = 0.0;
    int64_t capacity = 0;
    int64_t version = 0;
    int64_t next_ticket = 0;
    bool taken_this_version = false;  // the batch of the current version has been handed to the trainer
    struct Sample {
        int64_t ticket;
        int64_t init_version;
        int32_t state;        // 0 running, 1 interrupted (ABORT, waiting to resume), 2 complete
        int32_t resumes;      // times it was resumed under a newer policy
        uint64_t payload;
    };
    std::vector<Sample> live;  // outstanding samples, in order of begin()
    int64_t consumed = 0;
};

namespace {
roll_sample_buffer::Sample* find(roll_sample_buffer* b, int64_t ticket) {
    for (auto& s : b->live)
        if (s.ticket == ticket) return &s;
    return nullptr;
}
// A sample initiated at version v may still be consumed at version n iff n - v <= alpha.
bool due(const roll_sample_buffer* b, const roll_sample_buffer::Sample& s) {
    return (double)(b->version + 1 - s.init_version) > b->alpha;  // waiting one more version would be too old
}
}  // namespace

extern "C" int roll_sample_buffer_create(roll_sample_buffer** out, int32_t batch_size, double alpha) {
    if (!out) return roll::fail(ROLL_ERR_INVALID_ARG, "out is NULL");
    if (batch_size <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "batch_size must be > 0");
    if (!(alpha >= 0.0) || std::isinf(alpha)) return roll::fail(ROLL_ERR_INVALID_ARG, "alpha must be finite and >= 0");
    roll_sample_buffer* b = new (std::nothrow) roll_sample_buffer();
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "out of host memory");
    b->batch = batch_size;
    b->alpha = alpha;
    b->capacity = (int64_t)std::floor((1.0 + alpha) * (double)batch_size + 1e-9);
    *out = b;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_destroy(roll_sample_buffer* b) {
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "buffer is NULL");
    delete b;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_begin(roll_sample_buffer* b, int64_t* ticket, int64_t* init_version) {
    if (!b || !ticket) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL argument");
    const int64_t batches_ahead = (b->taken_this_version ? 1 : 0) + (int64_t)b->live.size() / b->batch;
    if ((double)batches_ahead > b->alpha + 1e-9 || (int64_t)b->live.size() >= b->capacity)
        return roll::fail(ROLL_ERR_BUFFER_FULL, "%zu samples outstanding: a new one would be consumed %lld versions from now, alpha is %g",
                          b->live.size(), (long long)batches_ahead, b->alpha);
    b->live.push_back({b->next_ticket, b->version, 0, 0, 0});
    *ticket = b->next_ticket++;
    if (init_version) *init_version = b->version;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_complete(roll_sample_buffer* b, int64_t ticket, uint64_t payload) {
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "buffer is NULL");
    auto* s = find(b, ticket);
    if (!s) return roll::fail(ROLL_ERR_INVALID_ARG, "unknown ticket %lld", (long long)ticket);
    if (s->state != 0) return roll::fail(ROLL_ERR_INVALID_ARG, "ticket %lld is not running", (long long)ticket);
    s->state = 2;
    s->payload = payload;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_abort(roll_sample_buffer* b, int64_t ticket) {
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "buffer is NULL");
    auto* s = find(b, ticket);
    if (!s) return roll::fail(ROLL_ERR_INVALID_ARG, "unknown ticket %lld", (long long)ticket);
    if (s->state != 0) return roll::fail(ROLL_ERR_INVALID_ARG, "ticket %lld is not running", (long long)ticket);
    s->state = 1;  // reclaimed: stays outstanding, keeps its initiating version
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_resume(roll_sample_buffer* b, int64_t ticket, int64_t* version_now) {
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "buffer is NULL");
    auto* s = find(b, ticket);
    if (!s) return roll::fail(ROLL_ERR_INVALID_ARG, "unknown ticket %lld", (long long)ticket);
    if (s->state != 1) return roll::fail(ROLL_ERR_INVALID_ARG, "ticket %lld was not interrupted", (long long)ticket);
    s->state = 0;
    s->resumes += 1;
    if (version_now) *version_now = b->version;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_take_batch(roll_sample_buffer* b, int64_t* tickets, int64_t* init_versions,
                                             uint64_t* payloads) {
    if (!b || !tickets) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL argument");
    if (b->taken_this_version)
        return roll::fail(ROLL_ERR_INVALID_ARG, "the batch of version %lld was already taken: advance the version first", (long long)b->version);
    int64_t complete = 0, due_total = 0, due_complete = 0;
    for (const auto& s : b->live) {
        const bool d = due(b, s);
        complete += s.state == 2;
        due_total += d;
        due_complete += d && s.state == 2;
    }
    if (due_complete < due_total)
        return roll::fail(ROLL_ERR_WOULD_BLOCK, "%lld samples are due but still generating", (long long)(due_total - due_complete));
    if (complete < b->batch)
        return roll::fail(ROLL_ERR_WOULD_BLOCK, "%lld of %d samples complete", (long long)complete, b->batch);
    if (due_total > b->batch)
        return roll::fail(ROLL_ERR_INVALID_ARG, "%lld samples are due, more than one batch: the freshness rule was already broken", (long long)due_total);
    // due first, then oldest initiating version (live is in begin order, so versions are non-decreasing)
    std::vector<size_t> pick;
    for (size_t i = 0; i < b->live.size(); ++i)
        if (due(b, b->live[i])) pick.push_back(i);
    for (size_t i = 0; i < b->live.size() && (int64_t)pick.size() < b->batch; ++i)
        if (!due(b, b->live[i]) && b->live[i].state == 2) pick.push_back(i);
    std::sort(pick.begin(), pick.end());
    for (size_t k = 0; k < pick.size(); ++k) {
        const auto& s = b->live[pick[k]];
        tickets[k] = s.ticket;
        if (init_versions) init_versions[k] = s.init_version;
        if (payloads) payloads[k] = s.payload;
    }
    for (size_t k = pick.size(); k-- > 0;) b->live.erase(b->live.begin() + (std::ptrdiff_t)pick[k]);
    b->consumed += b->batch;
    b->taken_this_version = true;
    return ROLL_OK;
}

extern "C" int roll_sample_buffer_advance_version(roll_sample_buffer* b) {
    if (!b) return roll::fail(ROLL_ERR_INVALID_ARG, "buffer is NULL");
    for (const auto& s : b->live)
        if (due(b, s))
            return roll::fail(ROLL_ERR_WOULD_BLOCK, "ticket %lld (version %lld) would become older than alpha", (long long)s.ticket,
                              (long long)s.init_version);
    b->version += 1;
    b->taken_this_version = false;
    return ROLL_OK;
}

extern "C" int64_t roll_sample_buffer_version(const roll_sample_buffer* b) { return b ? b->version : -1; }
extern "C" int64_t roll_sample_buffer_outstanding(const roll_sample_buffer* b) { return b ? (int64_t)b->live.size() : -1; }
extern "C" int64_t roll_sample_buffer_capacity(const roll_sample_buffer* b) { return b ? b->capacity : -1; }
