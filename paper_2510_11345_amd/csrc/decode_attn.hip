// Paged GQA decode attention for gfx950: ONE persistent stream-K kernel on the
// matrix cores; rows that were cut across waves are merged inside it.
//
// ROLL Flash (arXiv 2510.11345) Section 1: decoding is memory-bandwidth bound
// and response lengths are long-tailed; Section 4.2: one step over the whole
// running batch per loop iteration.  The kernel's only job is therefore to
// stream each live KV byte exactly once at HBM speed while rows of very
// different lengths share the chip evenly.
//
// Work decomposition (split-K over the flattened batch).  Row b with L_b tokens
// is ceil(L_b / 32) steps of 32 tokens; the rows' steps are laid end to end
// and cut into ranges of equal cost (a row's steps plus one for starting it:
// see Deal), one per persistent workgroup of four waves.  The four waves of a workgroup walk the SAME range of row steps, each
// for KV heads of its own (wave j: heads j, j + 4, ...; with fewer than four KV
// heads the range is cut again so that every wave has a part of one head).
// They run in step, so at any moment the workgroup reads the blocks of one page
// for four neighbouring heads, which lie next to each other in the pool: the
// memory system delivers 6.9-7.0 TB/s to such reads and 6.0-6.2 TB/s when the
// four waves read pages of their own (measured with equal rows, all else
// equal).  Every wave has the same share of the work whatever the length mix, a
// row longer than a range is cut across neighbouring workgroups, and for every
// head at most the first and the last row of a range are pieces; a wave writes
// a complete (row, head) stream straight to `out` and a piece (running max,
// sum, un-normalised output) to one of the two slots of its (range, head).
// Pieces are merged by whichever wave delivers the last one (an arrival counter
// per group of 16 neighbouring pieces, then one per stream when a stream has
// more than 16): no wave ever waits for another, so there is nothing to hang.
// The row prefix sums that locate a wave's first step are rebuilt in LDS by
// every workgroup (a few microseconds, no separate launch, no dependent
// global loads on the way to the first KV byte).  All G = Hq / Hkv query heads
// that share the KV head ride in one MFMA tile, so a KV byte is fetched once and
// used G times.
//
// The per-step arithmetic (S^T = K Q^T, online softmax, O^T += V^T P^T on the matrix cores) is
// shared with the prefill kernel and described where it is defined.
#include <cfloat>
#include <cmath>
#include <climits>
#include <cstddef>
#include <cstring>
#include <mutex>
#include <vector>

#include <type_traits>

#include "attn_core.h"
#include "attn_deal.h"
#include "common.h"
#include "kv_layout.h"
#include "kv_pool_internal.h"

namespace {

using namespace roll::attn;
static_assert(kDealStep == kStep, "the dealing and the kernel must agree on the step");

constexpr int kMaxBatch = 8192;    // rows whose prefix sums fit the LDS budget
constexpr int kMaxStreams = 65536; // batch * num_kv_heads: one arrival counter each
constexpr int kMergeGroup = 16;    // pieces merged by one wave at the first level
// Upper bound of persistent waves, used to size the workspace without touching the device:
// one workgroup on each of 256 compute units (a gfx950 device has no more).
constexpr int32_t kMaxPersistentWaves = kGroupWaves * 256;
// Tag that roll_decode_attn_workspace_init leaves in a workspace's header; the kernel refuses a
// buffer without it.
constexpr uint32_t kWorkspaceTag = 0x524F4C57u;

struct AttnParams {
    int32_t B, Hq, Hkv, G;
    int32_t Hs;       // page stride of the pools in head blocks (Hkv when dense)
    int32_t log2P, max_pages, num_pages;
    int32_t max_len;
    int32_t W;        // persistent waves launched
    int32_t out_f32;
    float scale_log2e;
};

// First words of a workspace.
struct WorkspaceHeader {
    int32_t grid_arrivals;  // workgroups of a fused step that have read the old lengths (zero between calls)
    uint32_t tag;           // kWorkspaceTag once prepared
    uint32_t refused;       // launches that found no tag and did nothing
};

struct Workspace {
    WorkspaceHeader* header;
    // zero between calls (roll_decode_attn_workspace_init, then every merger resets its counter)
    int32_t* group_arrivals;   // [kMaxSlots] indexed by the slot of the first piece of a group
    int32_t* stream_arrivals;  // [kMaxStreams] indexed by row * Hkv + kv head
    // scratch
    float2* part_ml;   // [slots * 16] (max in log2 units, sum) of a piece's heads: one 128-byte line per slot
    float* part_acc;   // [slots * G * D] un-normalised output of a piece
    float2* group_ml;  // [slots * 16] merged group of pieces, at the slot of the group's first piece
    float* group_acc;  // [slots * G * D]
    size_t header_bytes;
    size_t bytes;
};

__host__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Lays a workspace out for launches of up to `waves` persistent waves; with base == nullptr only
// the sizes are filled in.  The header does not depend on the shape
// (roll_decode_attn_workspace_init has none).
__host__ Workspace carve(void* base, int32_t Hkv, int32_t G, int32_t D, int32_t waves = kMaxPersistentWaves) {
    Workspace w{};
    const size_t slots = 2 * (size_t)max_ranges(waves, Hkv) * Hkv;
    size_t off = 0;
    auto take = [&](size_t bytes) -> char* {
        char* at = base ? (char*)base + off : nullptr;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.header = (WorkspaceHeader*)take(sizeof(WorkspaceHeader));
    w.group_arrivals = (int32_t*)take(sizeof(int32_t) * kMaxSlots);
    w.stream_arrivals = (int32_t*)take(sizeof(int32_t) * kMaxStreams);
    w.header_bytes = off;
    w.part_ml = (float2*)take(sizeof(float2) * slots * 16);
    w.part_acc = (float*)take(sizeof(float) * slots * G * D);
    w.group_ml = (float2*)take(sizeof(float2) * slots * 16);
    w.group_acc = (float*)take(sizeof(float) * slots * G * D);
    w.bytes = off;
    return w;
}

// Zeroes the header's words (counters included) and leaves the tag.
__global__ void prepare_header(uint32_t* dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = i == offsetof(WorkspaceHeader, tag) / 4 ? kWorkspaceTag : 0u;
}

// Built with -DROLL_ATTN_TIMELINE (paper_2510_11345_amd.build --timeline, a library of its own), every
// wave of attn_stream leaves eight 64-bit words in the buffer handed to roll_prof_attn_timeline:
// the constant 100 MHz clock at entry, after the row prefix is built, after its first step, after
// its last step, at exit; the steps it ran; its XCD; the streams it started.  The product build
// has none of this.
#ifdef ROLL_ATTN_TIMELINE
__device__ uint64_t* g_timeline = nullptr;
#define ROLL_TIMELINE(slot, value)                                                    \
    do {                                                                              \
        if (tl && lane == 0) tl[(size_t)w * 8 + (slot)] = (uint64_t)(value);          \
    } while (0)
#else
#define ROLL_TIMELINE(slot, value) do { } while (0)
#endif

// KV is read exactly once per step: a nontemporal load keeps it from displacing the
// page table, Q and the pieces in L2 (measured: +10 % on a plain streaming read).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int D>
struct WaveCtx {
    const uint4* __restrict__ k_pages;
    const uint4* __restrict__ v_pages;
    const int32_t* __restrict__ pt_row;
    int32_t h, Hkv, Hs, log2P, num_pages, max_pages, r, q;
    // Fused step only: the stream's newest token is not in the pages yet; its K row, V row,
    // position, page index and physical page.
    const uint4* __restrict__ k_new_row;
    const uint16_t* __restrict__ v_new_row;
    int32_t new_tok, new_pi, new_page;
};

// Extra kernel arguments of the fused step (allocator commit + K/V append + attention).
struct FusedArgs {
    int32_t n_delta;
    int32_t slot[roll::kMaxFusedDeltas];  // slot that was given a fresh page for its newest token
    int32_t page[roll::kMaxFusedDeltas];
    const uint4* k_new;                   // [B, Hkv, D] bf16: the newest token of every slot
    const uint4* v_new;
    int32_t* page_table_w;
    int32_t* seq_lens_w;
};
struct NoFusedArgs {};

// Physical pages of the (up to) two pages a 32-token step touches.
// NEWEST: the step holds the stream's newest token in a fused launch.
template <int D, bool NEWEST>
__device__ __forceinline__ void step_pages(const WaveCtx<D>& c, int32_t t0, int32_t& pgA, int32_t& pgB) {
    // A page index may lie past the row's end (the second page of a tail step, or a step
    // requested one ahead of the stream's last); its table entry is then stale or -1.  Reading
    // it is in bounds (clamped to the table row) and the id is clamped below, so the loads stay
    // inside the pool; the tokens are masked by the caller.  Not clamping to the row's own
    // last page keeps the row length off the address path.
    int32_t pa = t0 >> c.log2P;
    pa = pa > c.max_pages - 1 ? c.max_pages - 1 : pa;
    int32_t pb = (t0 + 16) >> c.log2P;
    pb = pb > c.max_pages - 1 ? c.max_pages - 1 : pb;
    pgA = c.pt_row[pa];
    pgB = c.pt_row[pb];
    pgA = pgA < 0 ? 0 : (pgA >= c.num_pages ? c.num_pages - 1 : pgA);
    pgB = pgB < 0 ? 0 : (pgB >= c.num_pages ? c.num_pages - 1 : pgB);
    if (NEWEST) {  // the table entry of the newest token's page may not be written yet
        if (pa == c.new_pi) pgA = c.new_page;
        if (pb == c.new_pi) pgB = c.new_page;
    }
}

// K: lane (r, q) reads, for tile tt and k-block kk, 8 head-dim elements 32kk+8q.. of
// token 8*(r>>2) + 4*tt + (r&3) of the step.  In the page's permuted token order that
// token sits at slot (r & 7) + 8 tt of page r >> 3 when P == 16, and at slot r + 16 tt of
// the step's 32-slot block otherwise: the 16 rows of a tile are contiguous, so one load
// instruction covers whole 128-byte lines.
// With NEWEST the lane that owns the newest token reads its row from k_new instead.
template <int D, bool NEWEST>
__device__ __forceinline__ void load_k(const WaveCtx<D>& c, int32_t t0, int32_t pgA, int32_t pgB, StepData<D>& s) {
    const int32_t P = 1 << c.log2P;
    const uint4* kbase[2];
    bool fresh[2] = {false, false};
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int32_t page = (P == 16 && c.r >= 8) ? pgB : pgA;
        const int32_t slot = P == 16 ? (c.r & 7) + 8 * tt : (t0 & (P - 1)) + c.r + 16 * tt;
        kbase[tt] = c.k_pages + (((int64_t)page * c.Hs + c.h) * (D / 8) + c.q) * P + slot;
        if (NEWEST) fresh[tt] = t0 + 8 * (c.r >> 2) + 4 * tt + (c.r & 3) == c.new_tok;
    }
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const uint4* src = kbase[tt] + (int64_t)kk * 4 * P;
            if (NEWEST && fresh[tt]) src = c.k_new_row + c.q + kk * 4;
            s.k[tt][kk] = load_stream(src);
        }
}

// V: lane (r, q) reads, for d-tile nt, the 8 tokens 8q..8q+7 of head-dim element 16nt+r.
template <int D>
__device__ __forceinline__ void load_v(const WaveCtx<D>& c, int32_t t0, int32_t pgA, int32_t pgB, StepData<D>& s) {
    const int32_t P = 1 << c.log2P;
    const int32_t page = c.q >= 2 ? pgB : pgA;
    const int32_t oct = ((t0 + 8 * c.q) & (P - 1)) >> 3;
    const uint4* base = c.v_pages + (((int64_t)page * c.Hs + c.h) * (P / 8) + oct) * D + c.r;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) s.v[nt] = load_stream(base + nt * 16);
}

// Fused launch, the step that holds a stream's newest token: the sixteen lanes of the token's
// octet put the token's element (fresh[nt] = v_new[16nt + r], fetched when the stream began)
// into the octets they have just read.
template <int D>
__device__ __forceinline__ void patch_newest_v(const WaveCtx<D>& c, int32_t t0, const uint32_t (&fresh)[D / 16],
                                               StepData<D>& s) {
    const int32_t j = c.new_tok - (t0 + 8 * c.q);
    if (j < 0 || j >= 8) return;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        uint32_t w[4] = {s.v[nt].x, s.v[nt].y, s.v[nt].z, s.v[nt].w};
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
            if (j == 2 * k2) w[k2] = (w[k2] & 0xFFFF0000u) | fresh[nt];
            if (j == 2 * k2 + 1) w[k2] = (w[k2] & 0x0000FFFFu) | (fresh[nt] << 16);
        }
        s.v[nt] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Raw scores of the step's 32 tokens for head r; the 8 a lane owns are tokens t0 + 8q + j.
// Tokens at or past `end` get -inf.
template <int D>
__device__ __forceinline__ void score_step(const WaveCtx<D>& c, const bf16x8_t (&qf)[D / 32],
                                           const StepData<D>& s, int32_t t0, int32_t end, float (&sv)[8]) {
    qk_scores<D>(qf, s, sv);
    if (t0 + kStep > end) {  // ragged tail of the row
        const int32_t first = t0 + 8 * c.q;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (first + j >= end) sv[j] = -INFINITY;
    }
}

// Online softmax update with the step's scores and O^T += V^T P^T.  Consumes the V registers.
// NEWEST: the step ends the row even when it is full (its newest token came from v_new).
// The running max stays finite: every processed step has a valid token.
template <int D, bool NEWEST>
__device__ __forceinline__ void accumulate_step(const WaveCtx<D>& c, const float (&sv)[8], StepData<D>& s,
                                                int32_t t0, int32_t end, float scale_log2e, WaveAcc<D>& a) {
    if (NEWEST || t0 + kStep > end) mask_v_tail<D>(s, end - (t0 + 8 * c.q));  // ragged tail
    softmax_pv<D>(sv, s, scale_log2e, a);
}

// Steps per row into LDS as an exclusive prefix, clamped lengths beside it, and the number of
// rows with tokens before each row.  pre and live have B + 1 entries, len has B.  All threads of
// the workgroup take part.  With grow, every row that holds tokens counts one more than the
// stored length (the token appended by the same launch).
__device__ void build_row_prefix(const int32_t* seq_lens, int32_t B, int32_t max_len, bool grow,
                                 int32_t* pre, int32_t* len, uint16_t* live, int32_t* s_wave_tot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;
    int32_t carry = 0, carry_live = 0;
    for (int32_t base = 0; base < B; base += nthreads) {
        const int32_t b = base + tid;
        int32_t L = 0;
        if (b < B) {
            L = seq_lens[b];
            if (grow && L > 0) ++L;
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
            len[b] = L;
        }
        const int32_t n = (L + kStep - 1) / kStep;
        int32_t incl = n;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        const unsigned long long live_mask = __ballot(n > 0);
        const int32_t live_before = (int32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(live_mask >> 32),
                                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)live_mask, 0u));
        if (lane == 63) {
            s_wave_tot[wave] = incl;
            s_wave_tot[kGroupWaves + wave] = (int32_t)__popcll(live_mask);
        }
        __syncthreads();
        int32_t before = carry, before_live = carry_live;
        for (int w = 0; w < wave; ++w) {
            before += s_wave_tot[w];
            before_live += s_wave_tot[kGroupWaves + w];
        }
        for (int w = 0; w < nwaves; ++w) {
            carry += s_wave_tot[w];
            carry_live += s_wave_tot[kGroupWaves + w];
        }
        if (b < B) {
            pre[b] = before + incl - n;
            live[b] = (uint16_t)(before_live + live_before);
        }
        __syncthreads();
    }
    if (tid == 0) {
        pre[B] = carry;
        live[B] = (uint16_t)carry_live;
    }
    __syncthreads();
}

// The last b in [0, n) with key(b) <= x, for a non-decreasing key with key(0) <= x < key(n): the
// interval is cut into (up to) 64 parts per round, lane l probing the start of part l + 1; the
// probes that hold are the first ones, so their count names the part to go on with.  The same
// result in every lane.
template <typename KeyFn>
__device__ __forceinline__ int32_t wave_last_row(int32_t n, int64_t x, KeyFn key, int32_t lane) {
    int32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int32_t stride = (hi - lo + 63) >> 6;
        const int32_t probe = lo + (lane + 1) * stride;
        const bool holds = probe < hi && key(probe) <= x;
        const int32_t t = (int32_t)__popcll(__ballot(holds));
        lo += t * stride;
        hi = lo + stride < hi ? lo + stride : hi;
    }
    return lo;
}

// Pieces travel between waves on different XCDs (each with its own L2) inside one kernel.
// They are written and read with relaxed device-scope atomic 8-byte accesses, which are
// coherent across the XCDs by themselves; the handshake is a device-scope atomic counter.
// That keeps the whole-L2 write-back / invalidate of a device-scope fence out of a kernel
// whose L2s are busy streaming KV.
__device__ __forceinline__ void coherent_store2(float* p, float a, float b) {
    const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
    __hip_atomic_store((uint64_t*)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x2_t coherent_load2(const float* p) {
    const uint64_t bits = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return f32x2_t{__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32))};
}

// A piece's un-normalised output in the workspace: G * D floats per slot, laid out for the wave
// that writes it, not by head: the 8-byte unit that lane (r, q) stores with its k-th instruction
// (k = 2 nt + half) sits at unit (4 k + q) G + r, so that one store instruction of the wave covers
// 32 G contiguous bytes, whole 32-byte sectors.  (By head, every instruction wrote half of each
// sector it touched, and these stores go through to memory one by one.)
__device__ __forceinline__ int64_t piece_unit(int64_t slot, int32_t G, int32_t D, int32_t r, int32_t q) {
    return slot * ((int64_t)G * D) + 2 * ((int64_t)q * G + r);
}

// Store a piece (un-normalised) at `slot` of a piece array; lane (r, q) owns head r, quads 4q.
// Called by the whole wave: the (max, sum) pairs of all sixteen tile rows go out as one 128-byte
// line (the rows past G hold nothing that is read back), the output units only for r < G.
template <int D>
__device__ __forceinline__ void store_piece(const WaveAcc<D>& a, float2* ml, float* acc, int64_t slot,
                                            int32_t G, int32_t r, int32_t q) {
    if (q == 0) coherent_store2((float*)(ml + slot * 16 + r), a.m, a.l);
    if (r >= G) return;
    float* dst = acc + piece_unit(slot, G, D, r, q);
    const int32_t stride = 8 * G;  // floats between a lane's consecutive units
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        coherent_store2(dst + (2 * nt) * stride, a.o[nt][0], a.o[nt][1]);
        coherent_store2(dst + (2 * nt + 1) * stride, a.o[nt][2], a.o[nt][3]);
    }
}

// Log-sum-exp merge of n pieces whose slots are slot_of(0..n-1); result stays un-normalised.
// The pieces are taken four at a time, with all loads of a batch requested before the first is
// used: the merging wave has nothing else to do meanwhile and is usually one of the last to
// finish, so the merge's latency is the kernel's.  Piece number own_idx (none if negative) is
// taken from `own` (registers) instead of memory; the arithmetic is the same either way, so the
// result does not depend on which wave merges.
template <int D, typename SlotFn>
__device__ __forceinline__ void merge_pieces(WaveAcc<D>& out_acc, const float2* ml, const float* acc,
                                             int32_t n, SlotFn slot_of, int32_t G, int32_t r, int32_t q,
                                             const WaveAcc<D>* own = nullptr, int32_t own_idx = -1) {
    constexpr int kBatch = 4;
    float M = -INFINITY, lsum = 0.f;
    f32x4_t o[D / 16];
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int32_t base = 0; base < n; base += kBatch) {
        f32x2_t m_l[kBatch], lo[kBatch][D / 16], hi[kBatch][D / 16];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            m_l[k] = f32x2_t{-INFINITY, 0.f};
            if (base + k == own_idx) {
                m_l[k] = f32x2_t{own->m, own->l};
#pragma unroll
                for (int nt = 0; nt < D / 16; ++nt) {
                    lo[k][nt] = f32x2_t{own->o[nt][0], own->o[nt][1]};
                    hi[k][nt] = f32x2_t{own->o[nt][2], own->o[nt][3]};
                }
            } else if (base + k < n) {
                const int64_t slot = slot_of(base + k);
                m_l[k] = coherent_load2((const float*)(ml + slot * 16 + r));
                const float* src = acc + piece_unit(slot, G, D, r, q);
                const int32_t stride = 8 * G;
#pragma unroll
                for (int nt = 0; nt < D / 16; ++nt) {
                    lo[k][nt] = coherent_load2(src + (2 * nt) * stride);
                    hi[k][nt] = coherent_load2(src + (2 * nt + 1) * stride);
                }
            } else {
#pragma unroll
                for (int nt = 0; nt < D / 16; ++nt) lo[k][nt] = hi[k][nt] = f32x2_t{0.f, 0.f};
            }
        }
        float Mb = M;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) Mb = fmaxf(Mb, m_l[k][0]);
        // every piece holds a valid token, so Mb is finite; exp2(-inf - Mb) = 0 drops the rest
        const float keep = __builtin_amdgcn_exp2f(M - Mb);
        lsum *= keep;
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) o[nt] *= keep;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const float wgt = __builtin_amdgcn_exp2f(m_l[k][0] - Mb);
            lsum += m_l[k][1] * wgt;
#pragma unroll
            for (int nt = 0; nt < D / 16; ++nt)
                o[nt] += f32x4_t{lo[k][nt][0], lo[k][nt][1], hi[k][nt][0], hi[k][nt][1]} * wgt;
        }
        M = Mb;
    }
    out_acc.m = M;
    out_acc.l = lsum;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) out_acc.o[nt] = o[nt];
}

// One arrival at a counter; returns true in every lane of the wave that arrived last.
// The wave first waits until its own piece stores have completed (they bypass the caches, so
// completed means visible to every XCD), then bumps the counter with a device-scope atomic.
// The last arriver resets the counter for the next call; nobody else touches it any more.
__device__ __forceinline__ bool arrive_last(int32_t* counter, int32_t expected, int32_t lane) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int32_t old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    asm volatile("" ::: "memory");
    if (old != expected - 1) return false;
    if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Physical page of the newest token (position L - 1) of `slot`: from the deltas when that
// token opened a page, else from the slot's page-table row.
__device__ __forceinline__ int32_t newest_page(const FusedArgs& fa, const int32_t* pt_row, int32_t slot,
                                               int32_t L, int32_t log2P, int32_t num_pages) {
    int32_t page = -1;
    if (((L - 1) & ((1 << log2P) - 1)) == 0)
        for (int32_t i = 0; i < fa.n_delta; ++i)
            if (fa.slot[i] == slot) page = fa.page[i];
    if (page < 0) page = pt_row[(L - 1) >> log2P];
    return page < 0 ? 0 : (page >= num_pages ? num_pages - 1 : page);
}

// FUSED: the launch is a whole decode step after the allocator's bookkeeping.  Lengths on the
// device are those before the step (every live row grows by one), the page-table deltas come as
// kernel arguments, and the newest token's K/V come from fa.k_new / fa.v_new.  The step that
// holds a stream's newest token runs as code of its own after the stream's loop: it takes that
// token's K row and V elements from k_new / v_new and its page from the arguments, so nothing in
// the launch reads what the launch writes.  The wave that ran that step writes the token into
// the pages once its attention work is done; workgroup 0 publishes the deltas; the lengths are
// written by the workgroup that is last to finish, when every workgroup has read the old ones.
// page_table and seq_lens stay __restrict__ although the launch writes both arrays through other
// pointers: no value it uses is read from an entry it writes.
template <int D, bool FUSED, bool F32OUT>
__global__ __launch_bounds__(kGroupWaves * 64) void attn_stream(
    const uint4* __restrict__ q16, const uint4* k_pages, const uint4* v_pages,
    const int32_t* __restrict__ page_table, const int32_t* __restrict__ seq_lens,
    void* __restrict__ out, WorkspaceHeader* header, int32_t* group_arrivals, int32_t* stream_arrivals,
    float2* part_ml, float* part_acc, float2* group_ml, float* group_acc, AttnParams prm,
    const typename std::conditional<FUSED, FusedArgs, NoFusedArgs>::type fa) {
    extern __shared__ int32_t lds[];
    int32_t* pre = lds;                  // [B + 1]
    int32_t* len = lds + prm.B + 1;      // [B]
    uint16_t* live = (uint16_t*)(lds + 2 * prm.B + 1);  // [B + 1] rows with tokens before row b
    __shared__ int32_t s_wave_tot[2 * kGroupWaves];
    // The workspace's tag, requested beside the lengths.  A buffer that was never prepared holds
    // arbitrary counters, with which cut rows would be merged too early or never: such a launch
    // writes nothing at all and leaves a mark for roll_decode_attn_workspace_check.
    const uint32_t tag = __hip_atomic_load(&header->tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#ifdef ROLL_ATTN_TIMELINE
    uint64_t* const tl = g_timeline;
    const uint64_t tl_entry = wall_clock64();
    uint64_t tl_first = 0, tl_steps = 0, tl_streams = 0;
#endif
    build_row_prefix(seq_lens, prm.B, prm.max_len, FUSED, pre, len, live, s_wave_tot);
    if (tag != kWorkspaceTag) {
        if (blockIdx.x == 0 && threadIdx.x == 0)
            __hip_atomic_fetch_add(&header->refused, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }

    const int32_t lane = threadIdx.x & 63;
    const int32_t w = blockIdx.x * kGroupWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t G = prm.G, Hkv = prm.Hkv;
    ROLL_TIMELINE(0, tl_entry);
    ROLL_TIMELINE(1, wall_clock64());

    if constexpr (FUSED) {
        if (blockIdx.x == 0)
            for (int32_t i = threadIdx.x; i < fa.n_delta; i += blockDim.x) {
                const int32_t slot = fa.slot[i];
                if (slot >= 0 && slot < prm.B && len[slot] > 0)
                    fa.page_table_w[(int64_t)slot * prm.max_pages + ((len[slot] - 1) >> prm.log2P)] = fa.page[i];
            }
    }

    // Rows without tokens give zeros; wave w of the launch clears rows w, w + W, ...
    for (int32_t b = w; b < prm.B; b += prm.W) {
        if (len[b] != 0) continue;
        const int64_t base = (int64_t)b * prm.Hq * D;
        for (int32_t e = lane * 4; e < prm.Hq * D; e += 256) {
            if (F32OUT) *(f32x4_t*)((float*)out + base + e) = f32x4_t{0.f, 0.f, 0.f, 0.f};
            else *(uint2*)((__bf16*)out + base + e) = make_uint2(0u, 0u);
        }
    }

    // Ranges of row steps and the (range, KV heads) of this wave: see the top of the file.
    const Deal deal(pre[prm.B], live[prm.B], prm.W, Hkv);
    const int32_t cut = ranges_cut(Hkv);
    const int32_t wj = w & (kGroupWaves - 1);
    const int32_t c = (int32_t)blockIdx.x * cut + (cut > 1 ? wj / Hkv : 0);
    const int32_t h_begin = cut > 1 ? wj % Hkv : wj;
    const int32_t h_stride = cut > 1 ? Hkv : kGroupWaves;  // cut > 1: one head per wave

    WaveCtx<D> ctx;
    ctx.k_pages = k_pages;
    ctx.v_pages = v_pages;
    ctx.Hkv = Hkv;
    ctx.Hs = prm.Hs;
    ctx.log2P = prm.log2P;
    ctx.num_pages = prm.num_pages;
    ctx.max_pages = prm.max_pages;
    ctx.r = lane & 15;
    ctx.q = lane >> 4;
    const int32_t rr = ctx.r < G ? ctx.r : 0;  // lanes of the padding heads shadow head 0, store nothing

    // The searches over the rows are done by the whole wave, 64 probes of LDS at a time (two or
    // three round trips instead of the eight to thirteen of a binary search): they stand between
    // the launch's start and the wave's first K/V byte.
    // The row that holds row step `item` (the last row b with pre[b] <= item; it is not empty).
    auto row_of = [&](int32_t item) -> int32_t {
        return wave_last_row(prm.B, (int64_t)item, [&](int32_t b) -> int64_t { return pre[b]; }, lane);
    };
    auto cost_pre = [&](int32_t b) -> int64_t { return roll::attn::cost_pre(pre, live, b); };
    auto first_step = [&](int32_t range) -> int32_t {
        if (range >= deal.NC) return pre[prm.B];
        const int64_t x = deal.boundary(range);
        return first_step_in_row(x, wave_last_row(prm.B, x, cost_pre, lane), pre, live);
    };
    const int32_t item0 = c < deal.NC ? first_step(c) : 0;
    const int32_t todo0 = c < deal.NC ? first_step(c + 1) - item0 : 0;

    for (int32_t h = h_begin; h < Hkv && todo0 > 0; h += h_stride) {
        int32_t todo = todo0;
        int32_t b = row_of(item0);
        int32_t n_b = pre[b + 1] - pre[b];
        int32_t s = item0 - pre[b];
        bool first_stream = true;
        // Delivers this wave's piece `mine` of row pb (the row spans the ranges c0..c1; piece i comes
        // from range c0 + i and sits in the first slot of (that range, h), except that c0 uses its
        // second slot when the row does not begin the range).  If every other piece of the group
        // has arrived already, this wave is the one that merges and its own piece never goes through
        // memory; that is the usual case for the piece that ends a range, whose partner began the
        // next range long ago.  Writes are what a ragged batch costs this kernel, and pieces are
        // most of them.
        auto deliver = [&](const WaveAcc<D>& mine, int32_t pb, bool begins) {
            const int32_t g0 = pre[pb], n_pb = pre[pb + 1] - g0;
            const int64_t x0 = cost_pre(pb) + kRowCost;  // the row's first step on the cost line
            const int32_t c0 = deal.owner(x0), c1 = deal.owner(x0 + (int64_t)(n_pb - 1) * kStepCost);
            const int32_t pieces = c1 - c0 + 1;
            // c0 begins with this row if it owns nothing of the row before: its boundary lies past
            // the first unit of that row's last step
            const int64_t slot0 = deal.slot(c0, h, Hkv, deal.boundary(c0) + kStepCost > cost_pre(pb));
            const int64_t out_idx = ((int64_t)pb * prm.Hq + (int64_t)h * G + rr) * D + 4 * ctx.q;
            const int32_t my_pi = c - c0;
            const int32_t gid = my_pi / kMergeGroup;
            const int32_t gfirst = gid * kMergeGroup;               // first piece of my group
            const int32_t gsize = min(kMergeGroup, pieces - gfirst);
            const int32_t ngroups = (pieces + kMergeGroup - 1) / kMergeGroup;
            // Slots are unique per piece, so the slot of a group's first piece names the group
            // (a range can end one row and begin the next: range numbers alone would collide).
            auto piece_slot = [&](int32_t pi) -> int64_t { return pi == 0 ? slot0 : deal.slot(c0 + pi, h, Hkv, true); };
            const int64_t group_slot = piece_slot(gfirst);
            int32_t* counter = group_arrivals + group_slot;

            WaveAcc<D> grp;
            bool merged = false;
            int32_t seen = 0;
            if (lane == 0) seen = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            seen = __builtin_amdgcn_readfirstlane(seen);
            if (seen == gsize - 1) {
                // Everybody else is here (an arrival follows the completion of the piece's stores),
                // and nobody touches the counter any more: reset it as a last arriver does.
                merge_pieces<D>(grp, part_ml, part_acc, gsize,
                                [&](int32_t i) -> int64_t { return piece_slot(gfirst + i); }, G, rr, ctx.q, &mine,
                                my_pi - gfirst);
                if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                merged = true;
            } else {
                store_piece<D>(mine, part_ml, part_acc, deal.slot(c, h, Hkv, begins), G, ctx.r, ctx.q);
                if (arrive_last(counter, gsize, lane)) {
                    merge_pieces<D>(grp, part_ml, part_acc, gsize,
                                    [&](int32_t i) -> int64_t { return piece_slot(gfirst + i); }, G, rr, ctx.q);
                    merged = true;
                }
            }
            if (!merged) return;
            if (ngroups == 1) {
                if (ctx.r < G) store_result_as<D, F32OUT>(grp, out, out_idx);
            } else {
                store_piece<D>(grp, group_ml, group_acc, group_slot, G, ctx.r, ctx.q);
                if (arrive_last(stream_arrivals + pb * Hkv + h, ngroups, lane)) {
                    WaveAcc<D> all;
                    merge_pieces<D>(all, group_ml, group_acc, ngroups,
                                    [&](int32_t j) -> int64_t { return piece_slot(j * kMergeGroup); }, G, rr, ctx.q);
                    if (ctx.r < G) store_result_as<D, F32OUT>(all, out, out_idx);
                }
            }
        };
        while (todo > 0) {
            const int32_t L = len[b];
            const int32_t cnt = min(todo, n_b - s);
            ctx.pt_row = page_table + (int64_t)b * prm.max_pages;
            ctx.h = h;
            if constexpr (FUSED) {
                ctx.k_new_row = fa.k_new + ((int64_t)b * Hkv + h) * (D / 8);
                ctx.v_new_row = (const uint16_t*)fa.v_new + ((int64_t)b * Hkv + h) * D;
                ctx.new_tok = L - 1;
                ctx.new_pi = (L - 1) >> prm.log2P;
                ctx.new_page = s + cnt == n_b ? newest_page(fa, ctx.pt_row, b, L, prm.log2P, prm.num_pages) : 0;
            }
            // The newest token's V elements this lane may need, fetched ahead of the stream's loads.
            uint32_t v_fresh[D / 16];
            if constexpr (FUSED) {
                if (s + cnt == n_b) {
#pragma unroll
                    for (int nt = 0; nt < D / 16; ++nt) v_fresh[nt] = ctx.v_new_row[16 * nt + ctx.r];
                }
            }

            // Q as the B operand: lane (r, q) holds head r, head-dim 32kk + 8q .. + 7; zero for r >= G.
            bf16x8_t qf[D / 32];
            {
                const uint4 zero = make_uint4(0, 0, 0, 0);
                const uint4* qrow = q16 + ((int64_t)b * prm.Hq + (int64_t)h * G + ctx.r) * (D / 8) + ctx.q;
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) qf[kk] = as_bf16x8(ctx.r < G ? qrow[kk * 4] : zero);
            }
            WaveAcc<D> acc;
#pragma unroll
            for (int nt = 0; nt < D / 16; ++nt) acc.o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            acc.m = -INFINITY;
            acc.l = 0.f;

            // In a fused launch the step that holds the stream's newest token runs as code of its
            // own after the loop, so that the loop is the same as in a plain launch.
            const bool has_newest = FUSED && s + cnt == n_b;
            const int32_t loop_end = s + cnt - (has_newest ? 1 : 0);
            {
                // The page ids of a step are requested one step early, through the scalar cache, so
                // that a miss there (one per 64-byte line of the table, every eighth step for
                // 16-token pages) does not sit between a step's arithmetic and the next loads; the
                // wave has no other wave on its SIMD to hide behind.  (Within the noise on c2.)
                int32_t pgA, pgB;
                step_pages<D, false>(ctx, s * kStep, pgA, pgB);
                for (int32_t i = s; i < loop_end; ++i) {
                    int32_t nxtA, nxtB;
                    step_pages<D, false>(ctx, (i + 1) * kStep, nxtA, nxtB);
                    StepData<D> sd;
                    load_k<D, false>(ctx, i * kStep, pgA, pgB, sd);
                    load_v<D>(ctx, i * kStep, pgA, pgB, sd);
                    float sv[8];
                    score_step<D>(ctx, qf, sd, i * kStep, L, sv);
                    accumulate_step<D, false>(ctx, sv, sd, i * kStep, L, prm.scale_log2e, acc);
#ifdef ROLL_ATTN_TIMELINE
                    if (tl_first == 0) tl_first = wall_clock64();
#endif
                    pgA = nxtA;
                    pgB = nxtB;
                }
            }
            if (has_newest) {
                const int32_t t0 = loop_end * kStep;
                StepData<D> sd;
                int32_t pgA, pgB;
                step_pages<D, FUSED>(ctx, t0, pgA, pgB);
                load_k<D, FUSED>(ctx, t0, pgA, pgB, sd);
                load_v<D>(ctx, t0, pgA, pgB, sd);
                float sv[8];
                score_step<D>(ctx, qf, sd, t0, L, sv);
                patch_newest_v<D>(ctx, t0, v_fresh, sd);
                accumulate_step<D, FUSED>(ctx, sv, sd, t0, L, prm.scale_log2e, acc);
            }

#ifdef ROLL_ATTN_TIMELINE
            tl_steps += (uint64_t)cnt;
            tl_streams += 1;
#endif
            // Finish the per-head sum across the four q-groups of the wave.
            acc.l = sum_over_q(acc.l);

            if (cnt == n_b) {  // the whole stream: normalise and write the result
                const int64_t out_idx = ((int64_t)b * prm.Hq + (int64_t)h * G + rr) * D + 4 * ctx.q;
                if (ctx.r < G) store_result_as<D, F32OUT>(acc, out, out_idx);
            } else {
                // A piece of a row that is cut across ranges: see deliver().
                deliver(acc, b, first_stream);
            }

            todo -= cnt;
            first_stream = false;
            s = 0;
            if (todo > 0) {  // the next row that has tokens
                do { ++b; } while (b < prm.B - 1 && pre[b + 1] == pre[b]);
                n_b = pre[b + 1] - pre[b];
            }
        }
    }

#ifdef ROLL_ATTN_TIMELINE
    ROLL_TIMELINE(2, tl_first);
    ROLL_TIMELINE(3, wall_clock64());
    ROLL_TIMELINE(5, tl_steps);
    ROLL_TIMELINE(7, tl_streams);
    {
        uint32_t xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        ROLL_TIMELINE(6, xcc & 0xF);
    }
#endif
    if constexpr (FUSED) {
        // Append pass, after the wave's attention work so that nothing waits for these stores:
        // the wave that owned a stream's last step writes that stream's newest token (the K and
        // V row of one KV head) into the pages.
        const int32_t P = 1 << prm.log2P;
        for (int32_t ah = h_begin; ah < Hkv && todo0 > 0; ah += h_stride) {
            int32_t atodo = todo0;
            int32_t ab = row_of(item0);
            int32_t an = pre[ab + 1] - pre[ab];
            int32_t as = item0 - pre[ab];
            while (atodo > 0) {
                const int32_t cnt = min(atodo, an - as);
                if (as + cnt == an) {
                    const int32_t L = len[ab];
                    const int32_t page = newest_page(fa, page_table + (int64_t)ab * prm.max_pages, ab, L, prm.log2P, prm.num_pages);
                    const int32_t pos = (L - 1) & (P - 1);
                    const int64_t row = (int64_t)ab * Hkv + ah;
                    if (lane < D / 8)
                        ((uint4*)k_pages)[(((int64_t)page * prm.Hs + ah) * (D / 8) + lane) * P + roll::k_slot(pos, P)] =
                            fa.k_new[row * (D / 8) + lane];
                    uint16_t* vdst = (uint16_t*)v_pages + ((((int64_t)page * prm.Hs + ah) * (P / 8) + pos / 8) * D) * 8 + pos % 8;
                    const uint16_t* vsrc = (const uint16_t*)fa.v_new + row * D;
#pragma unroll
                    for (int e = 0; e < D / 64; ++e) vdst[(int64_t)(lane + 64 * e) * 8] = vsrc[lane + 64 * e];
                }
                atodo -= cnt;
                as = 0;
                if (atodo > 0) {
                    do { ++ab; } while (ab < prm.B - 1 && pre[ab + 1] == pre[ab]);
                    an = pre[ab + 1] - pre[ab];
                }
            }
        }
    }

    if constexpr (FUSED) {
        // Every workgroup has read the old lengths long ago; the last one to get here writes the
        // new ones.  At the end of the wave's work the atomic's round trip delays nothing.
        if (threadIdx.x < 64 && arrive_last(&header->grid_arrivals, (int32_t)gridDim.x, lane))
            for (int32_t i = lane; i < prm.B; i += 64) fa.seq_lens_w[i] = len[i];
    }
    ROLL_TIMELINE(4, wall_clock64());
}

int validate(const roll_attn_desc* d) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->batch <= 0 || d->batch > kMaxBatch) return roll::fail(ROLL_ERR_INVALID_ARG, "batch must be in [1, %d]", kMaxBatch);
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads != 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "num_q_heads must be a positive multiple of num_kv_heads");
    if (d->num_q_heads / d->num_kv_heads > 16)
        return roll::fail(ROLL_ERR_INVALID_ARG, "GQA group size above 16 is not supported");
    if ((int64_t)d->batch * d->num_kv_heads > kMaxStreams)
        return roll::fail(ROLL_ERR_INVALID_ARG, "batch * num_kv_heads above %d", kMaxStreams);
    if (d->head_dim != 64 && d->head_dim != 128) return roll::fail(ROLL_ERR_INVALID_ARG, "head_dim must be 64 or 128");
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64");
    if (d->max_pages_per_seq <= 0 || d->num_pages <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq and num_pages must be > 0");
    if ((int64_t)d->max_pages_per_seq * d->page_size > (1 << 24))
        return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq * page_size above 2^24 tokens");
    // the kernel keeps the rows' step counts as 32-bit prefix sums
    if ((int64_t)d->batch * (((int64_t)d->max_pages_per_seq * d->page_size + kStep - 1) / kStep) > INT32_MAX)
        return roll::fail(ROLL_ERR_SEQ_TOO_LONG, "batch * ceil(max_pages_per_seq * page_size / %d) above 2^31 - 1 steps", kStep);
    if (d->out_dtype != ROLL_BF16 && d->out_dtype != ROLL_F32) return roll::fail(ROLL_ERR_INVALID_ARG, "out_dtype must be ROLL_BF16 or ROLL_F32");
    if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return roll::fail(ROLL_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    if (roll::page_stride_heads(d->page_stride, d->num_kv_heads, d->page_size, d->head_dim) == 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_stride must be 0 or a multiple of page_size * head_dim that holds all KV heads");
    return ROLL_OK;
}

// Persistent waves to launch: one workgroup (kGroupWaves waves, one per SIMD) on every compute
// unit of the current device.  Measured on c2 / c3 / c5: 3 to 4 waves per CU with 16 KiB in flight
// each already sit on the memory system's plateau; 8 per CU are 1-2 % slower and 2 per CU need
// double buffering to get there.  Fewer waves also mean fewer cut rows to merge.  No wave waits
// for another, so nothing depends on the workgroups being resident together: a workgroup that
// does not fit (LDS for the batch's prefix sums) fails the launch itself.
constexpr int kMaxDevices = 64;
int persistent_waves(int32_t* waves_out, int* device_out = nullptr) {
    static std::mutex mu;
    static int cu_count[kMaxDevices] = {0};
    int dev = 0;
    ROLL_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return roll::fail(ROLL_ERR_HIP, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (cu_count[dev] == 0) {
        int n = 0;
        ROLL_HIP_CHECK(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        if (n < 1) return roll::fail(ROLL_ERR_HIP, "device %d reports no compute units", dev);
        cu_count[dev] = n;
    }
    int32_t W = kGroupWaves * cu_count[dev];
    *waves_out = W > kMaxPersistentWaves ? kMaxPersistentWaves : W;
    if (device_out) *device_out = dev;
    return ROLL_OK;
}

// Profiling events of the calling thread (roll_prof_attn_events).
thread_local hipEvent_t t_ev_begin = nullptr, t_ev_end = nullptr;

}  // namespace

extern "C" size_t roll_decode_attn_workspace_bytes(const roll_attn_desc* d) {
    if (validate(d) != ROLL_OK) return 0;
    return carve(nullptr, d->num_kv_heads, d->num_q_heads / d->num_kv_heads, d->head_dim).bytes;
}

extern "C" int roll_decode_attn_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace || !roll::aligned(workspace, 256)) return roll::fail(ROLL_ERR_WORKSPACE, "workspace NULL or not 256-byte aligned");
    const Workspace ws = carve(workspace, 1, 1, 64);
    if (workspace_bytes < ws.header_bytes)
        return roll::fail(ROLL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.header_bytes);
    const size_t words = ws.header_bytes / 4;
    prepare_header<<<(unsigned)((words + 255) / 256), 256, 0, (hipStream_t)stream>>>((uint32_t*)workspace, words);
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}

extern "C" int roll_decode_attn_workspace_check(const void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace || !roll::aligned(workspace, 256)) return roll::fail(ROLL_ERR_WORKSPACE, "workspace NULL or not 256-byte aligned");
    const Workspace ws = carve(nullptr, 1, 1, 64);
    if (workspace_bytes < ws.header_bytes)
        return roll::fail(ROLL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.header_bytes);
    ROLL_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    std::vector<uint32_t> host(ws.header_bytes / 4);
    ROLL_HIP_CHECK(hipMemcpy(host.data(), workspace, ws.header_bytes, hipMemcpyDeviceToHost));
    WorkspaceHeader h;
    memcpy(&h, host.data(), sizeof h);
    if (h.tag != kWorkspaceTag)
        return roll::fail(ROLL_ERR_WORKSPACE, "workspace was never prepared (roll_decode_attn_workspace_init)");
    if (h.refused != 0)
        return roll::fail(ROLL_ERR_WORKSPACE, "%u launch(es) found the workspace unprepared and wrote no results", h.refused);
    size_t dirty = h.grid_arrivals != 0;
    for (size_t i = align_up(sizeof(WorkspaceHeader), 256) / 4; i < host.size(); ++i) dirty += host[i] != 0u;
    if (dirty != 0)
        return roll::fail(ROLL_ERR_WORKSPACE, "%zu arrival counter(s) are not zero: a launch on this workspace did not finish", dirty);
    return ROLL_OK;
}

extern "C" int roll_prof_attn_timeline(void* buffer, size_t buffer_bytes) {
#ifdef ROLL_ATTN_TIMELINE
    if (buffer && buffer_bytes < (size_t)kMaxPersistentWaves * 8 * sizeof(uint64_t))
        return roll::fail(ROLL_ERR_WORKSPACE, "timeline buffer too small: %zu < %zu bytes", buffer_bytes,
                          (size_t)kMaxPersistentWaves * 8 * sizeof(uint64_t));
    uint64_t* p = (uint64_t*)buffer;
    ROLL_HIP_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &p, sizeof p));
    return ROLL_OK;
#else
    (void)buffer;
    (void)buffer_bytes;
    return roll::fail(ROLL_ERR_INVALID_ARG, "this library was built without ROLL_ATTN_TIMELINE "
                                            "(python -m paper_2510_11345_amd.build --timeline builds one with it)");
#endif
}

extern "C" int roll_prof_attn_events(void* begin, void* end) {
    if ((begin == nullptr) != (end == nullptr)) return roll::fail(ROLL_ERR_INVALID_ARG, "begin and end must both be set or both NULL");
    t_ev_begin = (hipEvent_t)begin;
    t_ev_end = (hipEvent_t)end;
    return ROLL_OK;
}

extern "C" int roll_decode_attn_ranges(const roll_attn_desc* d, const int32_t* seq_lens_host, int32_t workgroups,
                                       int32_t* first_step_out, int32_t capacity, int32_t* num_ranges_out) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    if (!seq_lens_host || !first_step_out || !num_ranges_out) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (workgroups <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "workgroups must be > 0");
    const int32_t B = d->batch;
    const int64_t max_len = (int64_t)d->max_pages_per_seq * d->page_size;
    std::vector<int32_t> pre((size_t)B + 1);
    std::vector<uint16_t> live((size_t)B + 1);
    int64_t steps = 0;
    int32_t rows = 0;
    for (int32_t b = 0; b < B; ++b) {
        int64_t L = seq_lens_host[b];
        L = L < 0 ? 0 : (L > max_len ? max_len : L);
        pre[(size_t)b] = (int32_t)steps;
        live[(size_t)b] = (uint16_t)rows;
        steps += (L + kStep - 1) / kStep;
        rows += L > 0;
        if (steps > INT32_MAX) return roll::fail(ROLL_ERR_SEQ_TOO_LONG, "more than 2^31 steps of %d tokens in the batch", kStep);
    }
    pre[(size_t)B] = (int32_t)steps;
    live[(size_t)B] = (uint16_t)rows;
    int64_t waves = (int64_t)workgroups * kGroupWaves;
    if (waves > kMaxPersistentWaves) waves = kMaxPersistentWaves;
    const Deal deal((int32_t)steps, rows, (int32_t)waves, d->num_kv_heads);
    *num_ranges_out = deal.NC;
    if (capacity < deal.NC + 1)
        return roll::fail(ROLL_ERR_INVALID_ARG, "first_step_out holds %d entries, %d needed", capacity, deal.NC + 1);
    for (int32_t c = 0; c <= deal.NC; ++c) first_step_out[c] = first_step(deal, c, B, pre.data(), live.data());
    return ROLL_OK;
}

namespace {

// Argument checks and the launch shared by the entry points.  ws_of(W) hands over the laid-out
// scratch for a launch of W persistent waves, or fails.
template <typename WsFn>
int launch_attn(const void* q, const void* k_pages, const void* v_pages, const int32_t* page_table,
                const int32_t* seq_lens, void* out, const roll_attn_desc* d, WsFn ws_of, hipStream_t stream,
                FusedArgs* fused) {
    if (!q || !k_pages || !v_pages || !page_table || !seq_lens || !out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(q, 16) || !roll::aligned(k_pages, 16) || !roll::aligned(v_pages, 16) || !roll::aligned(out, 16) ||
        !roll::aligned(page_table, 4) || !roll::aligned(seq_lens, 4))
        return roll::fail(ROLL_ERR_INVALID_ARG, "q, k_pages, v_pages, out must be 16-byte aligned");
    const int32_t G = d->num_q_heads / d->num_kv_heads;
    int32_t W = 0;
    Workspace ws{};
    int rc = ws_of(&W, &ws);
    if (rc != ROLL_OK) return rc;
    W = W / kGroupWaves * kGroupWaves;

    const size_t lds = sizeof(int32_t) * (2 * (size_t)d->batch + 1) + sizeof(uint16_t) * ((size_t)d->batch + 2);
    AttnParams prm{};
    prm.B = d->batch;
    prm.Hq = d->num_q_heads;
    prm.Hkv = d->num_kv_heads;
    prm.G = G;
    prm.Hs = roll::page_stride_heads(d->page_stride, d->num_kv_heads, d->page_size, d->head_dim);
    prm.log2P = d->page_size == 16 ? 4 : (d->page_size == 32 ? 5 : 6);
    prm.max_pages = d->max_pages_per_seq;
    prm.num_pages = d->num_pages;
    prm.max_len = (int32_t)((int64_t)d->max_pages_per_seq * d->page_size);
    prm.W = W;
    prm.out_f32 = d->out_dtype == ROLL_F32;
    const float scale = d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / sqrtf((float)d->head_dim);
    prm.scale_log2e = scale * 1.44269504088896340736f;

    const unsigned grid = (unsigned)(W / kGroupWaves);
    if (t_ev_begin) ROLL_HIP_CHECK(hipEventRecord(t_ev_begin, stream));
#define ROLL_LAUNCH_ATTN(DIM, FUSED, F32, EXTRA)                                                              \
    attn_stream<DIM, FUSED, F32><<<grid, kGroupWaves * 64, lds, stream>>>(                                   \
        (const uint4*)q, (const uint4*)k_pages, (const uint4*)v_pages, page_table, seq_lens, out, ws.header,  \
        ws.group_arrivals, ws.stream_arrivals, ws.part_ml, ws.part_acc, ws.group_ml, ws.group_acc, prm, EXTRA)
#define ROLL_LAUNCH_ATTN_OUT(DIM, FUSED, EXTRA)                  \
    do {                                                         \
        if (prm.out_f32) ROLL_LAUNCH_ATTN(DIM, FUSED, true, EXTRA); \
        else ROLL_LAUNCH_ATTN(DIM, FUSED, false, EXTRA);            \
    } while (0)
    if (fused) {
        if (d->head_dim == 128) ROLL_LAUNCH_ATTN_OUT(128, true, *fused);
        else ROLL_LAUNCH_ATTN_OUT(64, true, *fused);
    } else {
        if (d->head_dim == 128) ROLL_LAUNCH_ATTN_OUT(128, false, NoFusedArgs{});
        else ROLL_LAUNCH_ATTN_OUT(64, false, NoFusedArgs{});
    }
#undef ROLL_LAUNCH_ATTN_OUT
#undef ROLL_LAUNCH_ATTN
    ROLL_HIP_CHECK(hipGetLastError());
    if (t_ev_end) ROLL_HIP_CHECK(hipEventRecord(t_ev_end, stream));
    return ROLL_OK;
}

// The scratch of a launch from a caller's workspace (sized for any launch, see carve).
struct CallerWorkspace {
    const roll_attn_desc* d;
    void* workspace;
    size_t workspace_bytes;
    int operator()(int32_t* W, Workspace* ws) const {
        if (!workspace || !roll::aligned(workspace, 256)) return roll::fail(ROLL_ERR_WORKSPACE, "workspace NULL or not 256-byte aligned");
        *ws = carve(workspace, d->num_kv_heads, d->num_q_heads / d->num_kv_heads, d->head_dim);
        if (workspace_bytes < ws->bytes)
            return roll::fail(ROLL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws->bytes);
        return persistent_waves(W);
    }
};

}  // namespace

extern "C" int roll_decode_attn(const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* page_table, const int32_t* seq_lens, void* out,
                                const roll_attn_desc* d, void* workspace, size_t workspace_bytes,
                                void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    return launch_attn(q, k_pages, v_pages, page_table, seq_lens, out, d, CallerWorkspace{d, workspace, workspace_bytes},
                       (hipStream_t)stream_v, nullptr);
}

extern "C" int roll_decode_step_attn(roll_kv_pool* pool, const void* k_new, const void* v_new, const void* q,
                                     void* k_pages, void* v_pages, void* out, const roll_attn_desc* d,
                                     void* workspace, size_t workspace_bytes, void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    if (!pool || !k_new || !v_new || !q || !k_pages || !v_pages || !out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(k_new, 16) || !roll::aligned(v_new, 16) || !roll::aligned(q, 16) || !roll::aligned(k_pages, 16) ||
        !roll::aligned(v_pages, 16) || !roll::aligned(out, 16))
        return roll::fail(ROLL_ERR_INVALID_ARG, "k_new, v_new, q, k_pages, v_pages, out must be 16-byte aligned");
    // the workspace is checked before the allocator's pending changes are touched, so that a
    // refused call leaves them pending
    {
        int32_t W;
        Workspace ws;
        rc = CallerWorkspace{d, workspace, workspace_bytes}(&W, &ws);
        if (rc != ROLL_OK) return rc;
    }
    hipStream_t stream = (hipStream_t)stream_v;
    roll::FusedPlan plan;
    rc = roll::plan_fused_step(pool, stream, &plan);
    if (rc != ROLL_OK) return rc;
    if (plan.num_slots != d->batch || plan.page_size != d->page_size || plan.max_pages != d->max_pages_per_seq ||
        plan.num_pages != d->num_pages)
        return roll::fail(ROLL_ERR_INVALID_ARG, "desc does not match the pool (slots %d, page size %d, max pages %d, pages %d)",
                          plan.num_slots, plan.page_size, plan.max_pages, plan.num_pages);
    const CallerWorkspace caller_ws{d, workspace, workspace_bytes};
    if (!plan.fusable) {
        // Not a plain decode step since the last commit (refills, first use, many new pages):
        // publish through the allocator's own kernel, then attend.
        rc = roll_kv_commit_append(pool, k_new, v_new, k_pages, v_pages, d->num_kv_heads, d->head_dim, d->page_stride,
                                   stream_v);
        if (rc != ROLL_OK) return rc;
        return launch_attn(q, k_pages, v_pages, plan.page_table_dev, plan.seq_lens_dev, out, d, caller_ws, stream,
                           nullptr);
    }
    FusedArgs fa{};
    fa.n_delta = plan.n_delta;
    for (int32_t i = 0; i < plan.n_delta; ++i) {
        fa.slot[i] = plan.slot[i];
        fa.page[i] = plan.page[i];
    }
    fa.k_new = (const uint4*)k_new;
    fa.v_new = (const uint4*)v_new;
    fa.page_table_w = plan.page_table_dev;
    fa.seq_lens_w = plan.seq_lens_dev;
    rc = launch_attn(q, k_pages, v_pages, plan.page_table_dev, plan.seq_lens_dev, out, d, caller_ws, stream, &fa);
    if (rc != ROLL_OK) return rc;
    roll::finish_fused_step(pool);
    return ROLL_OK;
}

// ---------------------------------------------------------------------------------------------
// roll_decode_attn_static: the plain attention launch on scratch that is part of the library's
// own device image, for callers that cannot allocate (HIP graph capture, serving loops and
// harnesses that forbid hipMalloc).  Each GPU the library runs on holds its own copy of the array
// until the process ends.  In host code the array's name is only a stand-in: its address on the
// current device comes from hipGetSymbolAddress, once per device, and only that pointer is ever
// handed to a kernel.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)48 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

struct StaticScratch {
    void* ptr = nullptr;    // address of `scratch` on this device
    bool prepared = false;  // its header has been zeroed and tagged by a kernel enqueued earlier
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mu;

// The scratch of a launch from the static array, laid out for exactly the waves the launch uses.
struct StaticWorkspace {
    const roll_attn_desc* d;
    hipStream_t stream;
    int operator()(int32_t* W, Workspace* ws) const {
        int dev = 0;
        int rc = persistent_waves(W, &dev);
        if (rc != ROLL_OK) return rc;
        const Workspace need = carve(nullptr, d->num_kv_heads, d->num_q_heads / d->num_kv_heads, d->head_dim, *W);
        if (need.bytes > kStaticScratchBytes)
            return roll::fail(ROLL_ERR_WORKSPACE,
                              "this shape needs %zu bytes of scratch, the static buffer holds %zu: use roll_decode_attn "
                              "with a workspace of the caller's", need.bytes, kStaticScratchBytes);
        std::lock_guard<std::mutex> lock(g_static_mu);
        StaticScratch& st = g_static[dev];
        if (!st.ptr) {
            void* p = nullptr;
            ROLL_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p || !roll::aligned(p, 256)) return roll::fail(ROLL_ERR_HIP, "static scratch has no usable device address");
            st.ptr = p;
        }
        if (!st.prepared) {
            // a fill kernel, not hipMemsetAsync: the call may be recorded into a graph
            const size_t words = need.header_bytes / 4;
            prepare_header<<<(unsigned)((words + 255) / 256), 256, 0, stream>>>((uint32_t*)st.ptr, words);
            ROLL_HIP_CHECK(hipGetLastError());
            st.prepared = true;
        }
        *ws = carve(st.ptr, d->num_kv_heads, d->num_q_heads / d->num_kv_heads, d->head_dim, *W);
        return ROLL_OK;
    }
};

}  // namespace

extern "C" int roll_decode_attn_static(const void* q, const void* k_pages, const void* v_pages,
                                       const int32_t* page_table, const int32_t* seq_lens, void* out,
                                       const roll_attn_desc* d, void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    return launch_attn(q, k_pages, v_pages, page_table, seq_lens, out, d, StaticWorkspace{d, (hipStream_t)stream_v},
                       (hipStream_t)stream_v, nullptr);
}
