// Page-table KV-cache allocator with slot free / refill, and the token writer
// that defines the two page layouts.
//
// ROLL Flash (arXiv 2510.11345), Section 4.2: requests join the running batch
// with ADD and leave it on completion or ABORT (their work is reclaimed and
// recomputed later); Section 5.1: a freed slot is handed the next prompt at
// once.  The paper leaves the cache to the engine; this is the allocator that
// makes "slot freed -> refilled" a constant-time host operation whose effect
// reaches the GPU as one small batched update per decode step.
//
// Design: all bookkeeping is host memory.  alloc / release only edit it and
// append (index, value) deltas; roll_kv_commit copies the current lengths and
// the deltas into a pinned staging block and enqueues one kernel that scatters
// them into the device tables.  A ring of staging blocks, each guarded by an
// event, lets the host run several steps ahead of the GPU without ever
// overwriting a block the GPU has not consumed.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"
#include "kv_layout.h"
#include "kv_pool_internal.h"

namespace {

constexpr int kRing = 8;
constexpr int kStageDeltas = 8192;  // (index, value) pairs per staging block

struct Stage {
    int32_t* host = nullptr;  // pinned; [num_slots lengths][num_slots append targets][2 * kStageDeltas deltas]
    int32_t* dev = nullptr;   // the same block as seen from the GPU
    hipEvent_t consumed = nullptr;
    bool in_flight = false;
};

__global__ void fill_i32(int32_t* dst, int64_t n, int32_t value) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

// stage = [lengths (num_slots)][append targets (num_slots)][pairs]; one thread per entry.
// With k_new set, the same launch also writes the newest token of every slot whose target
// (page * P + position in page, computed on the host from the same state) is >= 0.
__global__ void apply_updates(const int32_t* __restrict__ stage, int32_t* __restrict__ page_table,
                              int32_t* __restrict__ seq_lens, int32_t num_slots, int32_t copy_lens,
                              int32_t n_delta, int64_t table_elems, const uint4* __restrict__ k_new,
                              const uint4* __restrict__ v_new, uint4* __restrict__ k_pages,
                              uint16_t* __restrict__ v_pages, int32_t num_pages, int32_t P, int32_t Hkv,
                              int32_t D, int32_t Hs) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (copy_lens && i < num_slots) seq_lens[i] = stage[i];
    if (i < n_delta) {
        const int32_t idx = stage[2 * num_slots + 2 * i];
        const int32_t val = stage[2 * num_slots + 2 * i + 1];
        if (idx >= 0 && idx < table_elems) page_table[idx] = val;
    }
    if (k_new) {
        const int32_t d8n = D / 8;
        const int32_t items = num_slots * Hkv * d8n;
        if (i < items) {
            const int32_t c = i % d8n, h = (i / d8n) % Hkv, slot = i / (d8n * Hkv);
            const int32_t target = stage[num_slots + slot];
            if (target >= 0 && target / P < num_pages)
                roll::store_kv_slice(k_new[i], v_new[i], k_pages, v_pages, target / P, target % P, h, c, P, Hs, D);
        }
    }
}

// One thread per (token, kv head, 8-element slice of head_dim).
__global__ void append_tokens(const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
                              const int32_t* __restrict__ slots, const int32_t* __restrict__ positions,
                              const int32_t* __restrict__ seq_lens, int64_t n_items,
                              uint4* __restrict__ k_pages, uint16_t* __restrict__ v_pages,
                              const int32_t* __restrict__ page_table, int32_t max_pages,
                              int32_t num_pages, int32_t P, int32_t Hkv, int32_t D, int32_t Hs) {
    const int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= n_items) return;
    const int32_t d8n = D / 8;
    const int32_t c = (int32_t)(item % d8n);
    const int32_t h = (int32_t)((item / d8n) % Hkv);
    const int64_t tok = item / ((int64_t)d8n * Hkv);
    const int32_t slot = slots ? slots[tok] : (int32_t)tok;
    if (slot < 0) return;
    const int32_t pos = positions ? positions[tok] : seq_lens[slot] - 1;
    if (pos < 0) return;
    const int32_t pidx = pos / P;
    if (pidx >= max_pages) return;
    const int32_t page = page_table[(int64_t)slot * max_pages + pidx];
    if (page < 0 || page >= num_pages) return;
    roll::store_kv_slice(k_new[item], v_new[item], k_pages, v_pages, page, pos % P, h, c, P, Hs, D);
}

}  // namespace

struct roll_kv_pool {
    roll_kv_config cfg{};
    std::vector<int32_t> free_stack;  // free runs of `run` consecutive pages; back() is handed out next
    int32_t run = 1;                  // pages per run
    std::vector<int32_t> slot_pages;  // [num_slots * max_pages_per_seq]
    std::vector<int32_t> slot_npages;
    std::vector<int32_t> slot_len;
    std::vector<int32_t> pending;  // flat (index, value) pairs not yet on the device
    std::vector<uint32_t> stamp;   // per table entry: commit generation that last wrote it
    uint32_t generation = 0;
    std::vector<uint8_t> batch_seen;  // scratch of roll_kv_alloc_batch
    int32_t* page_table_dev = nullptr;
    int32_t* seq_lens_dev = nullptr;
    bool device_tables_initialised = false;
    // Lengths as the device holds them after the last commit (valid once one has happened).
    std::vector<int32_t> committed_len;
    bool committed_len_valid = false;
    int64_t fused_steps = 0;
    Stage ring[kRing];
    int ring_next = 0;
};

extern "C" int roll_kv_pool_create(roll_kv_pool** pool, const roll_kv_config* cfg,
                                   int32_t* page_table_dev, int32_t* seq_lens_dev) {
    if (!pool || !cfg) return roll::fail(ROLL_ERR_INVALID_ARG, "pool or cfg is NULL");
    if (cfg->num_pages <= 0 || cfg->num_slots <= 0 || cfg->max_pages_per_seq <= 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "num_pages, num_slots, max_pages_per_seq must be > 0");
    if (cfg->page_size != 16 && cfg->page_size != 32 && cfg->page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64 (got %d)", cfg->page_size);
    if ((page_table_dev == nullptr) != (seq_lens_dev == nullptr))
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_table_dev and seq_lens_dev must both be set or both NULL");
    if ((int64_t)cfg->num_slots * cfg->max_pages_per_seq > INT32_MAX)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page table larger than 2^31 entries");
    const int32_t run = cfg->run_pages == 0 ? 1 : cfg->run_pages;
    if (run != 1 && run != 2 && run != 4 && run != 8)
        return roll::fail(ROLL_ERR_INVALID_ARG, "run_pages must be 0, 1, 2, 4 or 8 (got %d)", cfg->run_pages);
    roll_kv_pool* p = new (std::nothrow) roll_kv_pool();
    if (!p) return roll::fail(ROLL_ERR_INVALID_ARG, "out of host memory");
    p->cfg = *cfg;
    p->run = run;
    const int32_t num_runs = cfg->num_pages / run;
    p->free_stack.resize(num_runs);
    for (int32_t i = 0; i < num_runs; ++i) p->free_stack[i] = num_runs - 1 - i;
    p->slot_pages.assign((size_t)cfg->num_slots * cfg->max_pages_per_seq, -1);
    p->slot_npages.assign(cfg->num_slots, 0);
    p->slot_len.assign(cfg->num_slots, 0);
    p->page_table_dev = page_table_dev;
    p->seq_lens_dev = seq_lens_dev;
    *pool = p;
    return ROLL_OK;
}

extern "C" int roll_kv_pool_destroy(roll_kv_pool* pool) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    int rc = ROLL_OK;
    for (Stage& s : pool->ring) {
        if (s.consumed) {
            if (s.in_flight && hipEventSynchronize(s.consumed) != hipSuccess) rc = ROLL_ERR_HIP;
            (void)hipEventDestroy(s.consumed);
        }
        if (s.host) (void)hipHostFree(s.host);
    }
    delete pool;
    if (rc != ROLL_OK) return roll::fail(rc, "hipEventSynchronize failed while destroying the pool");
    return ROLL_OK;
}

extern "C" int roll_kv_alloc(roll_kv_pool* pool, int32_t slot, int32_t n_tokens) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    const roll_kv_config& c = pool->cfg;
    if (slot < 0 || slot >= c.num_slots) return roll::fail(ROLL_ERR_SLOT_RANGE, "slot %d outside [0, %d)", slot, c.num_slots);
    if (n_tokens <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "n_tokens must be >= 1 (got %d)", n_tokens);
    const int64_t new_len = (int64_t)pool->slot_len[slot] + n_tokens;
    const int64_t need = (new_len + c.page_size - 1) / c.page_size;
    if (need > c.max_pages_per_seq)
        return roll::fail(ROLL_ERR_SEQ_TOO_LONG, "slot %d would need %lld pages (max %d)", slot, (long long)need, c.max_pages_per_seq);
    const int32_t have = pool->slot_npages[slot];
    const int32_t R = pool->run;
    const int64_t extra_runs = (need + R - 1) / R - (have + R - 1) / R;
    if (extra_runs > (int64_t)pool->free_stack.size())
        return roll::fail(ROLL_ERR_NO_PAGES, "slot %d needs %lld more runs of %d pages, %zu free", slot, (long long)extra_runs, R,
                          pool->free_stack.size());
    for (int32_t n = have; n < need; ++n) {
        const int32_t idx = slot * c.max_pages_per_seq + n;
        int32_t page;
        if (n % R == 0) {  // a new run
            page = pool->free_stack.back() * R;
            pool->free_stack.pop_back();
        } else {           // the next page of the slot's last run
            page = pool->slot_pages[idx - 1] + 1;
        }
        pool->slot_pages[idx] = page;
        pool->pending.push_back(idx);
        pool->pending.push_back(page);
    }
    pool->slot_npages[slot] = (int32_t)need;
    pool->slot_len[slot] = (int32_t)new_len;
    return ROLL_OK;
}

extern "C" int roll_kv_alloc_batch(roll_kv_pool* pool, const int32_t* slots, const int32_t* n_tokens,
                                   int32_t count) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    if (count < 0 || (count > 0 && (!slots || !n_tokens)))
        return roll::fail(ROLL_ERR_INVALID_ARG, "bad slots / n_tokens / count");
    const roll_kv_config& c = pool->cfg;
    // Pass 1: validate everything and count the pages needed; pass 2 cannot fail.
    std::vector<uint8_t>& seen = pool->batch_seen;
    seen.assign((size_t)c.num_slots, 0);
    int64_t extra_total = 0;
    for (int32_t i = 0; i < count; ++i) {
        const int32_t slot = slots[i];
        if (slot < 0 || slot >= c.num_slots) return roll::fail(ROLL_ERR_SLOT_RANGE, "slot %d outside [0, %d)", slot, c.num_slots);
        if (seen[slot]) return roll::fail(ROLL_ERR_INVALID_ARG, "slot %d appears twice in the batch", slot);
        seen[slot] = 1;
        if (n_tokens[i] <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "n_tokens must be >= 1 (got %d for slot %d)", n_tokens[i], slot);
        const int64_t need = ((int64_t)pool->slot_len[slot] + n_tokens[i] + c.page_size - 1) / c.page_size;
        if (need > c.max_pages_per_seq)
            return roll::fail(ROLL_ERR_SEQ_TOO_LONG, "slot %d would need %lld pages (max %d)", slot, (long long)need, c.max_pages_per_seq);
        extra_total += (need + pool->run - 1) / pool->run - (pool->slot_npages[slot] + pool->run - 1) / pool->run;
    }
    if (extra_total > (int64_t)pool->free_stack.size())
        return roll::fail(ROLL_ERR_NO_PAGES, "batch needs %lld more runs of %d pages, %zu free", (long long)extra_total, pool->run,
                          pool->free_stack.size());
    for (int32_t i = 0; i < count; ++i) {
        const int rc = roll_kv_alloc(pool, slots[i], n_tokens[i]);
        if (rc != ROLL_OK) return rc;  // unreachable after pass 1
    }
    return ROLL_OK;
}

extern "C" int roll_kv_release(roll_kv_pool* pool, int32_t slot) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    const roll_kv_config& c = pool->cfg;
    if (slot < 0 || slot >= c.num_slots) return roll::fail(ROLL_ERR_SLOT_RANGE, "slot %d outside [0, %d)", slot, c.num_slots);
    if (pool->slot_len[slot] == 0) return roll::fail(ROLL_ERR_SLOT_EMPTY, "slot %d holds no sequence", slot);
    const int32_t n = pool->slot_npages[slot];
    // Push in reverse so that an immediate re-alloc gets the pages back in the same order.
    for (int32_t i = n - 1; i >= 0; --i) {
        const int32_t idx = slot * c.max_pages_per_seq + i;
        if (i % pool->run == 0) pool->free_stack.push_back(pool->slot_pages[idx] / pool->run);
        pool->slot_pages[idx] = -1;
    }
    pool->slot_npages[slot] = 0;
    pool->slot_len[slot] = 0;
    return ROLL_OK;
}

extern "C" int roll_kv_free_pages(const roll_kv_pool* pool) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    return (int)pool->free_stack.size() * pool->run;
}

extern "C" int roll_kv_seq_len(const roll_kv_pool* pool, int32_t slot) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    if (slot < 0 || slot >= pool->cfg.num_slots) return roll::fail(ROLL_ERR_SLOT_RANGE, "slot %d outside [0, %d)", slot, pool->cfg.num_slots);
    return pool->slot_len[slot];
}

extern "C" int roll_kv_slot_pages(const roll_kv_pool* pool, int32_t slot, int32_t* pages_out, int32_t cap) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    if (slot < 0 || slot >= pool->cfg.num_slots) return roll::fail(ROLL_ERR_SLOT_RANGE, "slot %d outside [0, %d)", slot, pool->cfg.num_slots);
    const int32_t n = pool->slot_npages[slot];
    if (pages_out)
        for (int32_t i = 0; i < n && i < cap; ++i)
            pages_out[i] = pool->slot_pages[(size_t)slot * pool->cfg.max_pages_per_seq + i];
    return n;
}

static int acquire_stage(roll_kv_pool* pool, Stage** out) {
    Stage& s = pool->ring[pool->ring_next];
    pool->ring_next = (pool->ring_next + 1) % kRing;
    if (!s.host) {
        const size_t bytes = sizeof(int32_t) * (2 * (size_t)pool->cfg.num_slots + 2 * (size_t)kStageDeltas);
        ROLL_HIP_CHECK(hipHostMalloc((void**)&s.host, bytes, hipHostMallocDefault));
        ROLL_HIP_CHECK(hipHostGetDevicePointer((void**)&s.dev, s.host, 0));
        ROLL_HIP_CHECK(hipEventCreateWithFlags(&s.consumed, hipEventDisableTiming));
    }
    if (s.in_flight) {
        ROLL_HIP_CHECK(hipEventSynchronize(s.consumed));
        s.in_flight = false;
    }
    *out = &s;
    return ROLL_OK;
}

struct AppendArgs {
    const uint4* k_new = nullptr;
    const uint4* v_new = nullptr;
    uint4* k_pages = nullptr;
    uint16_t* v_pages = nullptr;
    int32_t Hkv = 0, D = 0;
    int32_t Hs = 0;  // page stride in head blocks
};

// Where the newest token of each live slot goes: page * P + position in page, -1 for an empty slot.
static void fill_append_targets(const roll_kv_pool* pool, int32_t* target) {
    const roll_kv_config& c = pool->cfg;
    for (int32_t slot = 0; slot < c.num_slots; ++slot) {
        const int32_t len = pool->slot_len[slot];
        target[slot] = len > 0 ? pool->slot_pages[(size_t)slot * c.max_pages_per_seq + (len - 1) / c.page_size] * c.page_size +
                                     (len - 1) % c.page_size
                               : -1;
    }
}

// First-use fill of the device table and de-duplication of the pending deltas.
static int prepare_commit(roll_kv_pool* pool, hipStream_t stream) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    if (!pool->page_table_dev) return roll::fail(ROLL_ERR_INVALID_ARG, "host-only pool has no device tables to commit to");
    const roll_kv_config& c = pool->cfg;
    const int64_t table_elems = (int64_t)c.num_slots * c.max_pages_per_seq;
    if (!pool->device_tables_initialised) {
        const int threads = 256;
        fill_i32<<<(unsigned)((table_elems + threads - 1) / threads), threads, 0, stream>>>(
            pool->page_table_dev, table_elems, -1);
        ROLL_HIP_CHECK(hipGetLastError());
        pool->device_tables_initialised = true;
    }
    // Keep only the newest value per table entry: the scatter kernel applies one block of
    // deltas in no particular order, so an entry must not appear twice.
    if (pool->stamp.empty()) pool->stamp.assign((size_t)table_elems, 0);
    if (++pool->generation == 0) {
        std::fill(pool->stamp.begin(), pool->stamp.end(), 0u);
        pool->generation = 1;
    }
    {
        std::vector<int32_t>& pd = pool->pending;
        size_t w = pd.size();
        for (size_t r = pd.size(); r >= 2; r -= 2) {
            const int32_t idx = pd[r - 2];
            if (pool->stamp[idx] == pool->generation) continue;
            pool->stamp[idx] = pool->generation;
            w -= 2;
            pd[w] = idx;
            pd[w + 1] = pd[r - 1];
        }
        pd.erase(pd.begin(), pd.begin() + (std::ptrdiff_t)w);
    }
    return ROLL_OK;
}

static int commit_impl(roll_kv_pool* pool, void* stream_v, const AppendArgs& ap) {
    hipStream_t stream = (hipStream_t)stream_v;
    int rc0 = prepare_commit(pool, stream);
    if (rc0 != ROLL_OK) return rc0;
    const roll_kv_config& c = pool->cfg;
    const int64_t table_elems = (int64_t)c.num_slots * c.max_pages_per_seq;
    const size_t n_pairs = pool->pending.size() / 2;
    size_t done = 0;
    bool first = true;
    while (first || done < n_pairs) {
        Stage* s = nullptr;
        int rc = acquire_stage(pool, &s);
        if (rc != ROLL_OK) return rc;
        const int32_t batch = (int32_t)std::min<size_t>(kStageDeltas, n_pairs - done);
        // Lengths go with the last block so that they never run ahead of their pages.
        const bool last = done + batch >= n_pairs;
        const bool append = last && ap.k_new != nullptr;
        if (last) std::memcpy(s->host, pool->slot_len.data(), sizeof(int32_t) * c.num_slots);
        if (append) fill_append_targets(pool, s->host + c.num_slots);
        if (batch > 0)
            std::memcpy(s->host + 2 * c.num_slots, pool->pending.data() + 2 * done, sizeof(int32_t) * 2 * batch);
        const int threads = 256;
        int32_t n = std::max(last ? c.num_slots : 0, batch);
        if (append) n = std::max(n, c.num_slots * ap.Hkv * (ap.D / 8));
        apply_updates<<<(n + threads - 1) / threads, threads, 0, stream>>>(
            s->dev, pool->page_table_dev, pool->seq_lens_dev, c.num_slots, last ? 1 : 0, batch, table_elems,
            append ? ap.k_new : nullptr, ap.v_new, ap.k_pages, ap.v_pages, c.num_pages, c.page_size, ap.Hkv,
            ap.D, ap.Hs);
        ROLL_HIP_CHECK(hipGetLastError());
        ROLL_HIP_CHECK(hipEventRecord(s->consumed, stream));
        s->in_flight = true;
        done += batch;
        first = false;
    }
    pool->pending.clear();
    pool->committed_len = pool->slot_len;
    pool->committed_len_valid = true;
    return ROLL_OK;
}

extern "C" int roll_kv_commit(roll_kv_pool* pool, void* stream) { return commit_impl(pool, stream, AppendArgs{}); }

int roll::plan_fused_step(roll_kv_pool* pool, hipStream_t stream, roll::FusedPlan* plan) {
    int rc = prepare_commit(pool, stream);
    if (rc != ROLL_OK) return rc;
    const roll_kv_config& c = pool->cfg;
    plan->num_slots = c.num_slots;
    plan->max_pages = c.max_pages_per_seq;
    plan->num_pages = c.num_pages;
    plan->page_size = c.page_size;
    plan->page_table_dev = pool->page_table_dev;
    plan->seq_lens_dev = pool->seq_lens_dev;
    plan->n_delta = 0;
    plan->fusable = 0;
    const size_t n_pairs = pool->pending.size() / 2;
    if (!pool->committed_len_valid || n_pairs > (size_t)roll::kMaxFusedDeltas) return ROLL_OK;
    for (int32_t slot = 0; slot < c.num_slots; ++slot) {
        const int32_t was = pool->committed_len[slot];
        if (pool->slot_len[slot] != was + (was > 0 ? 1 : 0)) return ROLL_OK;
    }
    for (size_t i = 0; i < n_pairs; ++i) {
        const int32_t idx = pool->pending[2 * i], slot = idx / c.max_pages_per_seq;
        const int32_t len = pool->slot_len[slot];
        if (len <= 0 || idx != slot * c.max_pages_per_seq + (len - 1) / c.page_size || (len - 1) % c.page_size != 0)
            return ROLL_OK;
        plan->slot[i] = slot;
        plan->page[i] = pool->pending[2 * i + 1];
    }
    plan->n_delta = (int32_t)n_pairs;
    plan->fusable = 1;
    return ROLL_OK;
}

void roll::finish_fused_step(roll_kv_pool* pool) {
    pool->pending.clear();
    pool->committed_len = pool->slot_len;
    ++pool->fused_steps;
}

extern "C" int64_t roll_kv_fused_steps(const roll_kv_pool* pool) {
    if (!pool) return roll::fail(ROLL_ERR_INVALID_ARG, "pool is NULL");
    return pool->fused_steps;
}

extern "C" int roll_kv_commit_append(roll_kv_pool* pool, const void* k_new, const void* v_new, void* k_pages,
                                     void* v_pages, int32_t num_kv_heads, int32_t head_dim, int64_t page_stride,
                                     void* stream) {
    if (!k_new || !v_new || !k_pages || !v_pages) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(k_new, 16) || !roll::aligned(v_new, 16) || !roll::aligned(k_pages, 16) || !roll::aligned(v_pages, 16))
        return roll::fail(ROLL_ERR_INVALID_ARG, "k_new, v_new, k_pages, v_pages must be 16-byte aligned");
    if (head_dim <= 0 || head_dim % 8 != 0 || num_kv_heads <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "bad shape");
    if (pool && (int64_t)pool->cfg.num_pages * pool->cfg.page_size > INT32_MAX)
        return roll::fail(ROLL_ERR_INVALID_ARG, "pool above 2^31 tokens");
    AppendArgs ap;
    ap.k_new = (const uint4*)k_new;
    ap.v_new = (const uint4*)v_new;
    ap.k_pages = (uint4*)k_pages;
    ap.v_pages = (uint16_t*)v_pages;
    ap.Hkv = num_kv_heads;
    ap.D = head_dim;
    ap.Hs = pool ? roll::page_stride_heads(page_stride, num_kv_heads, pool->cfg.page_size, head_dim) : num_kv_heads;
    if (ap.Hs == 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_stride must be 0 or a multiple of page_size * head_dim that holds all KV heads");
    return commit_impl(pool, stream, ap);
}

extern "C" int roll_kv_append_tokens(const void* k_new, const void* v_new, const int32_t* slots,
                                     const int32_t* positions, const int32_t* seq_lens,
                                     int32_t n_tokens, void* k_pages,
                                     void* v_pages, const int32_t* page_table, int32_t max_pages_per_seq,
                                     int32_t num_pages, int32_t page_size, int32_t num_kv_heads,
                                     int32_t head_dim, int64_t page_stride, void* stream) {
    if (n_tokens < 0) return roll::fail(ROLL_ERR_INVALID_ARG, "n_tokens < 0");
    if (n_tokens == 0) return ROLL_OK;
    if (!k_new || !v_new || !k_pages || !v_pages || !page_table)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!positions && !seq_lens)
        return roll::fail(ROLL_ERR_INVALID_ARG, "positions and seq_lens are both NULL");
    if (!roll::aligned(k_new, 16) || !roll::aligned(v_new, 16) || !roll::aligned(k_pages, 16) || !roll::aligned(v_pages, 16))
        return roll::fail(ROLL_ERR_INVALID_ARG, "k_new, v_new, k_pages, v_pages must be 16-byte aligned");
    if (page_size != 16 && page_size != 32 && page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64");
    if (head_dim <= 0 || head_dim % 8 != 0 || num_kv_heads <= 0 || max_pages_per_seq <= 0 || num_pages <= 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "bad shape");
    const int32_t Hs = roll::page_stride_heads(page_stride, num_kv_heads, page_size, head_dim);
    if (Hs == 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_stride must be 0 or a multiple of page_size * head_dim that holds all KV heads");
    const int64_t items = (int64_t)n_tokens * num_kv_heads * (head_dim / 8);
    const int threads = 256;
    append_tokens<<<(unsigned)((items + threads - 1) / threads), threads, 0, (hipStream_t)stream>>>(
        (const uint4*)k_new, (const uint4*)v_new, slots, positions, seq_lens, items, (uint4*)k_pages,
        (uint16_t*)v_pages, page_table, max_pages_per_seq, num_pages, page_size, num_kv_heads, head_dim, Hs);
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}
