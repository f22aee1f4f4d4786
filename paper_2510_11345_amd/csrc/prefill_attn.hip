// Chunked prefill attention into pages for gfx950.
//
// ROLL Flash (arXiv 2510.11345) Section 4.2: a request that joins the running batch (ADD, or a
// slot refilled by queue scheduling, Section 5.1.1) is prefilled before it is decoded step by
// step.  A chunk is a run of consecutive prompt tokens of one slot.  The entry point first
// writes the chunk tokens' K/V into the slot's pages (one small launch), then every chunk token
// attends causally over its slot's tokens 0 .. its own position, read from the pages in the
// two layouts the decode kernel streams.
//
// Unlike decoding this is a dense contraction: the query tokens of one head share every K/V
// byte, and the G query heads of a KV head share it again.  A wave's work is a unit: a span of
// 32 query tokens of a chunk for one query head, the tokens held as the columns of two MFMA
// tiles.  A chunk's units of one KV head, span after span and head after head, are dealt out U to
// a workgroup (7 computing waves and one that copies for a large launch, whatever G is: a
// workgroup's units may lie in several spans).  Each 32-token step of K and V is
// copied once per workgroup from the pages into LDS in 16-byte pieces with global_load_lds (the
// page layouts are already the A-operand layouts; the pieces are ordered so that consecutive
// lanes read consecutive pieces and the LDS reads are conflict free), into a ring of tiles with
// the copies of several steps in flight.  The per-step arithmetic is the decode kernel's with two
// differences: the mask is per column (column r sees tokens up to the position of query token r),
// and the softmax reference is handled lazily, because here instruction issue, not memory, is
// what the matrix cores wait for.
//
// What bounds the kernel is how fast a SIMD issues instructions: a matrix instruction holds the
// SIMD's vector issue port for about two thirds of the time the matrix core needs for it, a vector
// instruction of another kind fits in the rest only in part, a wave issues at most one
// instruction every eight cycles or so, and a branch on a vector result waits for the wave's
// matrix instructions in flight.  Workgroups of 8 waves (up to 8 query heads per KV head) with a
// bf16 result therefore run a loop built around that: spare waves do all the copying, the computing waves
// run the three parts of a step (scores, softmax, PV) of three consecutive steps side by side in
// one straight-line stretch, and the softmax reference is fixed after the first step and verified
// once at the end (a workgroup that fails the check repeats its block in the exact loop, which
// is also the loop of fp32 results).
#include <cmath>
#include <type_traits>

#include "attn_core.h"
#include "common.h"
#include "kv_layout.h"

namespace {

using namespace roll::attn;

constexpr int kTile = 16;         // query tokens per MFMA column tile
constexpr int kCopyWaves = 8;     // waves of a workgroup; where no wave is set aside for it, all of them copy K/V
constexpr int kCopyThreads = 64 * kCopyWaves;
constexpr int kComputeUnits = 256;   // of an MI355X (only how many query tokens a workgroup takes depends on it)
constexpr int kTiles = 4;         // LDS ring: the step in use and three steps of copies in flight
constexpr int kAhead = kTiles - 1;
// A row sum at or above this after the loop that never moves the softmax reference (or a NaN)
// sends the workgroup through the exact loop: probabilities up to 2^40 times those of the
// reference are harmless, beyond that products with V could overflow.
constexpr float kSumLimit = 1.0995116e12f;   // 2^40

// Built with -DROLL_ATTN_TIMELINE (paper_2510_11345_amd.build --timeline, a library of its own), wave 0
// of every workgroup of prefill_attn that stores a result leaves eight 64-bit words in the buffer
// handed to roll_prof_prefill_timeline: the constant 100 MHz clock at entry, when its block is
// found, before the first and after the last iteration of the step loop, after its stores; the
// hardware id (XCC_ID << 32 | HW_ID); its steps; 1.  The product build has none of this.
#ifdef ROLL_ATTN_TIMELINE
__device__ uint64_t* g_pf_timeline = nullptr;
__device__ uint32_t g_pf_timeline_blocks = 0;
#define ROLL_PF_STAMP(var) var = wall_clock64()
#else
#define ROLL_PF_STAMP(var) do { } while (0)
#endif

struct PrefillParams {
    int32_t C, T, Hq, Hkv, G;
    int32_t U;   // units per workgroup: a unit is (span of 32 or 16 query tokens, query head of the group)
    int32_t Hs;  // page stride of the pools in head blocks (Hkv when dense)
    int32_t log2P, max_pages, num_pages, num_slots;
    int32_t out_f32;
    float scale_log2e;
};

// The chunk that holds token t: the last c with chunk_offset[c] <= t.
__device__ __forceinline__ int32_t chunk_of_token(const int32_t* __restrict__ chunk_offset, int32_t C, int32_t t) {
    int32_t lo = 0, hi = C;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (chunk_offset[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// Writes the chunk tokens' K and V into the pages.  Tokens whose slot, position or page is out
// of range are skipped.  The first k_blocks workgroups write K: one thread per (token, KV head,
// 8 head-dim elements), a 16-byte store each, a wave taking 16 tokens x 4 pieces.  The others write V, whose layout keeps 8
// consecutive positions of one head-dim element together: one wave per (octet of positions of
// a chunk, KV head) gathers the (up to) 8 tokens' elements row by row and stores 16 bytes per
// head-dim element; an octet that the chunk covers only in part is written element by element
// so that the positions outside the chunk keep what they hold.
__global__ __launch_bounds__(256) void append_chunks(
    const uint4* __restrict__ k_new, const uint16_t* __restrict__ v_new, const int32_t* __restrict__ chunk_slot,
    const int32_t* __restrict__ chunk_start, const int32_t* __restrict__ chunk_offset, uint4* __restrict__ k_pages,
    uint4* __restrict__ v_pages, const int32_t* __restrict__ page_table, PrefillParams prm, int32_t D,
    int32_t k_blocks) {
    const int32_t P = 1 << prm.log2P;
    if ((int32_t)blockIdx.x < k_blocks) {
        // A wave takes 16 consecutive tokens x 4 consecutive pieces of a head: its loads are 16 runs of
        // 64 bytes, its stores (a page keeps the tokens of a piece side by side) 4 runs of 256 bytes
        // where the tokens share a page, instead of 64 pieces of 16 bytes in 64 different lines.
        const int32_t d8n = D / 8, per_tok = prm.Hkv * d8n, per_tok4 = per_tok >> 2;
        const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
        const int32_t lane = threadIdx.x & 63;
        const int64_t t16 = group / per_tok4;
        const int32_t t = (int32_t)(t16 * 16 + (lane >> 2)), rem = (int32_t)(group - t16 * per_tok4) * 4 + (lane & 3);
        if (t >= prm.T) return;
        const int64_t item = (int64_t)t * per_tok + rem;
        const uint4 piece = k_new[item];   // asked for before the lookups below, not after them
        const int32_t c = chunk_of_token(chunk_offset, prm.C, t);
        const int32_t slot = chunk_slot[c], pos = chunk_start[c] + (t - chunk_offset[c]);
        if (slot < 0 || slot >= prm.num_slots || pos < 0 || (pos >> prm.log2P) >= prm.max_pages) return;
        const int32_t page = page_table[(int64_t)slot * prm.max_pages + (pos >> prm.log2P)];
        if (page < 0 || page >= prm.num_pages) return;
        k_pages[(((int64_t)page * prm.Hs + rem / d8n) * d8n + rem % d8n) * P + roll::k_slot(pos & (P - 1), P)] = piece;
        return;
    }
    // V: which (chunk, octet of it) is this wave's?  Octets are numbered chunk after chunk; the
    // wave counts those of 64 chunks at a time.
    const int32_t lane = threadIdx.x & 63;
    const int32_t wave_ordinal = ((int32_t)blockIdx.x - k_blocks) * (int32_t)(blockDim.x >> 6) + (int32_t)(threadIdx.x >> 6);
    const int32_t waves_per_unit = D / 64;   // a wave covers 64 head-dim elements
    const int32_t unit = wave_ordinal / waves_per_unit, d = (wave_ordinal % waves_per_unit) * 64 + lane;
    const int32_t wanted = unit / prm.Hkv, h = unit % prm.Hkv;
    int32_t c = -1, k = 0, carry = 0;
    for (int32_t base = 0; base < prm.C && c < 0; base += 64) {
        const int32_t cc = base + lane;
        int32_t n_oct = 0;
        if (cc < prm.C) {
            const int32_t n = chunk_offset[cc + 1] - chunk_offset[cc], st = chunk_start[cc];
            if (n > 0 && st >= 0) n_oct = ((st + n + 7) >> 3) - (st >> 3);
        }
        int32_t incl = n_oct;
#pragma unroll
        for (int dd = 1; dd < 64; dd <<= 1) {
            const int32_t v = __shfl_up(incl, dd);
            if (lane >= dd) incl += v;
        }
        const int32_t first = carry + incl - n_oct;
        const uint64_t hit = __ballot(wanted >= first && wanted < first + n_oct);
        if (hit) {
            const int32_t src = __ffsll((unsigned long long)hit) - 1;
            c = base + src;
            k = wanted - __shfl(first, src);
        }
        carry += __shfl(incl, 63);
    }
    if (c < 0) return;   // past the last octet
    const int32_t slot = chunk_slot[c], start = chunk_start[c], n = chunk_offset[c + 1] - chunk_offset[c];
    const int32_t pos0 = ((start >> 3) + k) << 3;
    const int32_t lo = pos0 > start ? pos0 : start, hi = pos0 + 8 < start + n ? pos0 + 8 : start + n;
    if (slot < 0 || slot >= prm.num_slots || (pos0 >> prm.log2P) >= prm.max_pages) return;
    const int32_t page = page_table[(int64_t)slot * prm.max_pages + (pos0 >> prm.log2P)];
    if (page < 0 || page >= prm.num_pages) return;
    uint4* dst = v_pages + (((int64_t)page * prm.Hs + h) * (P / 8) + ((pos0 & (P - 1)) >> 3)) * D + d;
    const int64_t t_lo = (int64_t)chunk_offset[c] + (lo - start);   // the token at position lo
    if (hi - lo == 8) {   // a whole octet: the eight loads go out together
        const uint16_t* src = v_new + (t_lo * prm.Hkv + h) * D + d;
        const int64_t per_token = (int64_t)prm.Hkv * D;
        uint32_t val[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) val[j] = src[j * per_token];
        *dst = make_uint4(val[0] | (val[1] << 16), val[2] | (val[3] << 16), val[4] | (val[5] << 16), val[6] | (val[7] << 16));
    } else {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        for (int32_t pos = lo; pos < hi; ++pos) {
            const uint32_t val = v_new[((t_lo + (pos - lo)) * prm.Hkv + h) * D + d];
            const int32_t j = pos - pos0;
            w[j >> 1] |= val << ((j & 1) * 16);
        }
        uint16_t* dst16 = (uint16_t*)dst;
        for (int32_t pos = lo; pos < hi; ++pos) {
            const int32_t j = pos - pos0;
            dst16[j] = (uint16_t)(w[j >> 1] >> ((j & 1) * 16));
        }
    }
}

// LDS tile of one step (uint4 units): K [D/8][32 token slots of the step], then V [4 octets][D].
// Each of the kCopyThreads copying threads moves kPerThread 16-byte pieces per step, the same
// number in every copying wave, so that a wave can wait for "all but the youngest n steps" of
// its copies with one s_waitcnt vmcnt.
template <int D>
struct CopyPlan {
    static constexpr int kPieces = D * 8;   // (D/8) * 32 + 4 * D
    static constexpr int kPerThread = kPieces / kCopyThreads;
    static_assert(kPieces % kCopyThreads == 0, "pieces must divide evenly over the copying threads");
};

// Copies one step's K and V from the pages into an LDS tile with global_load_lds_dwordx4:
// each lane's 16 bytes go straight from memory to tile[wave-uniform base + lane] without
// passing through registers, asynchronously (the wave waits on vmcnt before the barrier that
// publishes the tile).  Called by all threads; the first kCopyThreads do the work.
struct StepPages { int32_t a, b; };   // physical pages of the (up to) two pages a step touches

// pt_row must be wave-uniform so that the page ids come through the scalar cache and do not
// share the counter of the copies.  Ids are clamped into the pool.
__device__ __forceinline__ StepPages step_page_ids(const int32_t* __restrict__ pt_row, int32_t t0, int32_t log2P,
                                                   int32_t max_pages, int32_t num_pages) {
    int32_t pa = t0 >> log2P, pb = (t0 + 16) >> log2P;
    pb = pb > max_pages - 1 ? max_pages - 1 : pb;   // a second page past the row's end is masked later
    int32_t pgA = pt_row[pa], pgB = pt_row[pb];
    pgA = pgA < 0 ? 0 : (pgA >= num_pages ? num_pages - 1 : pgA);
    pgB = pgB < 0 ? 0 : (pgB >= num_pages ? num_pages - 1 : pgB);
    return StepPages{pgA, pgB};
}

// What a copying thread keeps for the pieces it moves every step: the address of each piece in
// page 0 at step offset 0 (pool, KV head, place inside the page's head block), whether the piece
// lies in the step's second page (16-token pages), and how far a token of step offset inside a
// larger page moves it (uint4 units: 1 for a K piece, D/8 for a V piece).
template <int D>
struct CopySrc {
    const uint4* base[CopyPlan<D>::kPerThread];
    uint32_t per_token[CopyPlan<D>::kPerThread];
    bool second[CopyPlan<D>::kPerThread];
};

template <int D>
__device__ __forceinline__ CopySrc<D> copy_sources(const uint4* __restrict__ k_pages, const uint4* __restrict__ v_pages,
                                                   int32_t h, int32_t log2P) {
    const int32_t P = 1 << log2P;
    CopySrc<D> cs;
#pragma unroll
    for (int i = 0; i < CopyPlan<D>::kPerThread; ++i) {
        const int32_t idx = (threadIdx.x & (kCopyThreads - 1)) + i * kCopyThreads;
        if (idx < (D / 8) * 32) {
            // LDS order of the 32 token slots of a K row: the 16 slots that the lanes r = 0..15 of
            // MFMA tile tt read sit next to each other at 16 tt + r (256 contiguous bytes, all 64
            // banks once).  With 16-token pages those are the slots 8 tt .. 8 tt + 7 of the step's
            // first page and of its second page; with larger pages the page order is that order.
            const int32_t d8 = idx >> 5, pos = idx & 31;
            const int32_t s32 = P == 16 ? 16 * ((pos >> 3) & 1) + (pos & 7) + 8 * (pos >> 4) : pos;
            cs.second[i] = P == 16 && s32 >= 16;
            cs.base[i] = k_pages + ((int64_t)h * (D / 8) + d8) * P + (P == 16 ? (s32 & 15) : s32);
            cs.per_token[i] = 1u;
        } else {
            const int32_t j = idx - (D / 8) * 32, oct = j / D, d = j - oct * D;
            cs.second[i] = P == 16 && oct >= 2;
            cs.base[i] = v_pages + ((int64_t)h * (P / 8) + (P == 16 ? (oct & 1) : oct)) * D + d;
            cs.per_token[i] = (uint32_t)(D / 8);
        }
    }
    return cs;
}

// Copies one step's K and V from the pages into an LDS tile with global_load_lds_dwordx4.  Called
// by all threads; the first kCopyThreads do the work.  page_stride: uint4 units between pages
// (the same for K and V blocks).
template <int D>
__device__ __forceinline__ void copy_step(uint4* tile, const CopySrc<D>& cs, StepPages pg, int32_t t0, int32_t log2P,
                                          int64_t page_stride) {
    if (threadIdx.x >= kCopyThreads) return;
    const int32_t wave_base = (int32_t)(threadIdx.x & ~63u);
    const uint32_t in_page = (uint32_t)t0 & ((1u << log2P) - 1u);   // 0 with 16-token pages
    // The two page offsets are wave-uniform (scalar multiplies); a lane only picks one of them.
    const uint64_t offA = (uint64_t)(uint32_t)pg.a * (uint64_t)page_stride, offB = (uint64_t)(uint32_t)pg.b * (uint64_t)page_stride;
    const uint32_t a_lo = __builtin_amdgcn_readfirstlane((uint32_t)offA), a_hi = __builtin_amdgcn_readfirstlane((uint32_t)(offA >> 32));
    const uint32_t b_lo = __builtin_amdgcn_readfirstlane((uint32_t)offB), b_hi = __builtin_amdgcn_readfirstlane((uint32_t)(offB >> 32));
#pragma unroll
    for (int i = 0; i < CopyPlan<D>::kPerThread; ++i) {
        const uint32_t lo = cs.second[i] ? b_lo : a_lo, hi = cs.second[i] ? b_hi : a_hi;
        const uint4* src = cs.base[i] + (int64_t)(((uint64_t)hi << 32) | lo) + in_page * cs.per_token[i];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(tile + i * kCopyThreads + wave_base),
                                         16, 0, 0);
    }
}

// All of this wave's copies have landed in LDS except those of the youngest STEPS steps, and
// its own LDS reads have returned.  (s_waitcnt immediate of gfx9: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 left at its maximum, lgkmcnt 11:8 = 0.)
template <int D, int STEPS>
__device__ __forceinline__ void copies_landed_but() {
    constexpr int n = STEPS * CopyPlan<D>::kPerThread;
    static_assert(n < 64, "vmcnt field");
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | (7 << 4));
}

// The loop of a copying wave (workgroups with spare waves: the last NCP waves copy, wave cw of them
// here).  Lane cl = 64 cw + lane of the copying lanes moves the pieces cl, cl + 64 NCP, .. of a
// step's LDS tile, K pieces first, then V pieces.  What depends on the lane (the token slot of a K
// piece and, with 16-token pages, its page; the head-dim element of a V piece) is kept from before
// the loop; what depends on the piece is the same for the whole wave and, with the page size
// and NCP known to the compiler, an immediate.  One barrier after the first three steps' copies,
// then one per step, as in the computing waves.
template <int D, int LOG2P, int NCP>
__device__ __forceinline__ void copier_loop(uint4* tile0, uint4* tile1, uint4* tile2, uint4* tile3,
                                            const uint4* __restrict__ k_pages, const uint4* __restrict__ v_pages,
                                            const int32_t* __restrict__ pt_row, int32_t h, int32_t cw, int32_t lane,
                                            int32_t n_steps, int64_t page_stride, int32_t max_pages, int32_t num_pages) {
    constexpr int P = 1 << LOG2P;
    constexpr int kKPieces = (D / 8) * 32, kVPieces = 4 * D, kStride = 64 * NCP;
    constexpr int nk = kKPieces / kStride, nv = kVPieces / kStride;
    static_assert(nk >= 1 && nv >= 1 && (nk + nv) < 64, "pieces per lane");
    const int32_t cl = cw * 64 + lane;
    const int32_t pos = cl & 31;
    const int32_t s32 = P == 16 ? 16 * ((pos >> 3) & 1) + (pos & 7) + 8 * (pos >> 4) : pos;   // LDS order of a K row: see copy_sources
    const bool k_second = P == 16 && s32 >= 16;
    const uint4* k_lane = k_pages + ((int64_t)h * (D / 8) + (cl >> 5)) * P + (P == 16 ? (s32 & 15) : s32);
    const uint32_t v_lane = (uint32_t)(cl & (D - 1));
    const int32_t v_oct_of_wave = __builtin_amdgcn_readfirstlane(cl / D);
    const uint4* v_head = v_pages + (int64_t)h * (P / 8) * D;
    const int32_t last_t0 = (n_steps - 1) * kStep;
    auto ids_of = [&](int32_t step) {
        return step_page_ids(pt_row, min(step * kStep, last_t0), LOG2P, max_pages, num_pages);
    };
    auto copy_all = [&](int32_t step, StepPages pg) {
        const int32_t t0 = min(step * kStep, last_t0);
        uint4* tl = (step & 3) == 0 ? tile0 : (step & 3) == 1 ? tile1 : (step & 3) == 2 ? tile2 : tile3;
        uint4* dst = tl + cw * 64;
        const uint32_t in_page = (uint32_t)t0 & (uint32_t)(P - 1);   // 0 with 16-token pages
        const uint64_t offA = (uint64_t)(uint32_t)pg.a * (uint64_t)page_stride;
        const uint64_t offB = (uint64_t)(uint32_t)pg.b * (uint64_t)page_stride;
        const uint32_t a_lo = __builtin_amdgcn_readfirstlane((uint32_t)offA), a_hi = __builtin_amdgcn_readfirstlane((uint32_t)(offA >> 32));
        const uint32_t b_lo = __builtin_amdgcn_readfirstlane((uint32_t)offB), b_hi = __builtin_amdgcn_readfirstlane((uint32_t)(offB >> 32));
        const uint32_t lo = k_second ? b_lo : a_lo, hi = k_second ? b_hi : a_hi;
        const uint4* k_src = k_lane + (int64_t)(((uint64_t)hi << 32) | lo) + in_page;
#pragma unroll
        for (int ik = 0; ik < nk; ++ik)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(k_src + ik * (kStride >> 5) * P),
                                             (__attribute__((address_space(3))) void*)(dst + ik * kStride), 16, 0, 0);
#pragma unroll
        for (int iv = 0; iv < nv; ++iv) {
            const int32_t oct = (iv * kStride) / D + v_oct_of_wave;
            const int32_t d_extra = (iv * kStride) & (D - 1);
            const bool second = P == 16 && oct >= 2;
            const int32_t oct_in_page = P == 16 ? (oct & 1) : oct + (int32_t)(in_page >> 3);
            const uint4* v_base = v_head + (int64_t)(second ? offB : offA) + oct_in_page * D + d_extra;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(v_base + v_lane),
                                             (__attribute__((address_space(3))) void*)(dst + kKPieces + iv * kStride), 16, 0, 0);
        }
    };
    // All of this wave's copies but those of the youngest step have landed.
    auto landed_but_one = [&]() {
        constexpr int n = nk + nv;
        __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | (7 << 4) | (0xF << 8));
    };
    // The copying wave shares its SIMD with a computing wave that started before it and would
    // otherwise win every issue slot; its few instructions per step go first.
    __builtin_amdgcn_s_setprio(3);
    // The page ids of the first four steps in one round trip, then the copies back to back; in the
    // loop the ids come one step early.
    const StepPages pg0 = ids_of(0), pg1 = ids_of(1), pg2 = ids_of(2);
    StepPages pg_ahead = ids_of(kAhead);
    copy_all(0, pg0);
    copy_all(1, pg1);
    copy_all(2, pg2);
    landed_but_one();
    __builtin_amdgcn_s_barrier();
    for (int32_t s = 0; s < n_steps; ++s) {
        const StepPages pg = pg_ahead;
        pg_ahead = ids_of(s + kAhead + 1);
        copy_all(s + kAhead, pg);
        landed_but_one();
        __builtin_amdgcn_s_barrier();
    }
}

// Workgroups of 8 waves (the register budget follows from it).  QT: column tiles (16 query tokens
// each) per wave; every K/V piece read from LDS is used for all of them.  F32OUT: fp32 result, P
// split in two bf16 parts; else bf16 result, P rounded once.
template <int D, int QT, bool F32OUT>
__global__ __launch_bounds__(kCopyThreads) void prefill_attn(
    const uint4* __restrict__ q16, const uint4* __restrict__ k_pages, const uint4* __restrict__ v_pages,
    const int32_t* __restrict__ page_table, const int32_t* __restrict__ chunk_slot,
    const int32_t* __restrict__ chunk_start, const int32_t* __restrict__ chunk_offset,
    void* __restrict__ out, PrefillParams prm) {
    static_assert(kTiles == 4 && kAhead == 3, "the step loop is written out for four tiles");
    __shared__ uint4 tile0[CopyPlan<D>::kPieces], tile1[CopyPlan<D>::kPieces], tile2[CopyPlan<D>::kPieces],
        tile3[CopyPlan<D>::kPieces];
    __shared__ int32_t s_meta[8], s_found, s_redo;

    // Which (chunk, query block) is this workgroup's?  Blocks are numbered chunk after chunk;
    // the workgroups take them from the last one down, so that within a prompt the blocks
    // with the longest prefixes start first.  Wave 0 counts the blocks of 64 chunks at a time.
    constexpr int kSpan = kTile * QT;          // query tokens per wave
    // A chunk's units, span after span and head after head within a span, are dealt out U to a
    // workgroup; a chunk of n tokens has this many workgroups:
    auto blocks_of = [&](int32_t n) { return (((n + kSpan - 1) / kSpan) * prm.G + prm.U - 1) / prm.U; };
    const int32_t h = blockIdx.x % prm.Hkv;
    const int32_t wanted_from_end = blockIdx.x / prm.Hkv;
    const int32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#ifdef ROLL_ATTN_TIMELINE
    uint64_t tl_entry, tl_found, tl_loop = 0, tl_done = 0;
#endif
    ROLL_PF_STAMP(tl_entry);
    // (What the search finds goes to the other waves through LDS together with the chunk's slot,
    // start and offset, read in the same round trip as the lengths: every dependent trip to memory
    // before the first product is time in which the compute unit does nothing, about a
    // microsecond each.)
    if (wave == 0) {
        if (lane == 0) { s_found = 0; s_redo = 0; }
        if (prm.C <= 64) {   // one round of 64 lanes holds all chunks: their arrays are read once
            const bool in = lane < prm.C;
            const int32_t o0 = in ? chunk_offset[lane] : 0, o1 = in ? chunk_offset[lane + 1] : 0;
            const int32_t sl = in ? chunk_slot[lane] : 0, st = in ? chunk_start[lane] : 0;
            const int32_t n = o1 - o0, nb = blocks_of(n);
            int32_t incl = nb;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int32_t v = __shfl_up(incl, d);
                if (lane >= d) incl += v;
            }
            const int32_t wanted = __shfl(incl, 63) - 1 - wanted_from_end, first = incl - nb;
            if (wanted >= first && wanted < first + nb) {
                s_meta[0] = sl;
                s_meta[1] = st;
                s_meta[2] = o0;
                s_meta[3] = n;
                s_meta[4] = wanted - first;
                s_found = 1;
            }
        } else {
            int32_t total = 0;
            for (int32_t base = 0; base < prm.C; base += 64) {
                const int32_t c = base + lane;
                const int32_t n = c < prm.C ? chunk_offset[c + 1] - chunk_offset[c] : 0;
                int32_t incl = blocks_of(n);
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int32_t v = __shfl_up(incl, d);
                    if (lane >= d) incl += v;
                }
                total += __shfl(incl, 63);
            }
            const int32_t wanted = total - 1 - wanted_from_end;
            int32_t carry = 0;
            for (int32_t base = 0; base < prm.C && wanted >= 0; base += 64) {
                const int32_t c = base + lane;
                const int32_t o0 = c < prm.C ? chunk_offset[c] : 0, o1 = c < prm.C ? chunk_offset[c + 1] : 0;
                const int32_t n = o1 - o0, nb = blocks_of(n);
                int32_t incl = nb;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int32_t v = __shfl_up(incl, d);
                    if (lane >= d) incl += v;
                }
                const int32_t first = carry + incl - nb;
                if (wanted >= first && wanted < first + nb) {
                    s_meta[0] = chunk_slot[c];
                    s_meta[1] = chunk_start[c];
                    s_meta[2] = o0;
                    s_meta[3] = n;
                    s_meta[4] = wanted - first;
                    s_found = 1;
                }
                carry += __shfl(incl, 63);
            }
        }
    }
    __syncthreads();
    if (!s_found) return;
    ROLL_PF_STAMP(tl_found);
    // (wave-uniform by construction; saying so keeps everything derived from them in scalar registers)
    const int32_t slot = __builtin_amdgcn_readfirstlane(s_meta[0]);
    const int32_t chunk_first = __builtin_amdgcn_readfirstlane(s_meta[1]);
    const int32_t chunk_off = __builtin_amdgcn_readfirstlane(s_meta[2]);
    const int32_t n_c = __builtin_amdgcn_readfirstlane(s_meta[3]);
    const int32_t qb = __builtin_amdgcn_readfirstlane(s_meta[4]);
    // The workgroup's units u0 .. u0 + U - 1 lie in the spans u0 / G .. (u0 + U - 1) / G of the chunk
    // (the last workgroup of a chunk may run out of units before it runs out of waves).
    const int32_t u0 = prm.U * qb, spans_c = (n_c + kSpan - 1) / kSpan;
    const int32_t span_last = min((u0 + prm.U - 1) / prm.G, spans_c - 1);
    if (slot < 0 || slot >= prm.num_slots || chunk_first < 0) return;
    int32_t kv_end = chunk_first + min(n_c, kSpan * (span_last + 1));   // tokens the last query sees
    const int32_t cap = prm.max_pages << prm.log2P;
    kv_end = kv_end > cap ? cap : kv_end;
    const int32_t n_steps = (kv_end + kStep - 1) / kStep;
    const int32_t* pt_row = page_table + (int64_t)slot * prm.max_pages;

    // Wave w computes unit u0 + w: whatever the number of query heads per KV head, U waves of the
    // workgroup (and both issue slots of the SIMDs they sit on) have work.  The workgroup's units
    // may lie in different spans; all of them run the steps of the last span, those past a
    // span's own last token masked like the diagonal.
    const int32_t wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int32_t span = (u0 + wave_s) / prm.G, head = (u0 + wave_s) - span * prm.G;
    const int32_t tq0_w = chunk_off + kSpan * span, pos0_w = chunk_first + kSpan * span;   // the wave's first query token, its position
    const int32_t nq_w = min(kSpan, n_c - kSpan * span);                                    // the wave's query tokens
    const int32_t r = lane & 15, q = lane >> 4;
    const bool computes = wave_s < prm.U && span < spans_c;   // the other waves only copy (or wait)
    int32_t pq[QT];                                           // newest position column r of tile c sees
    bf16x8_t qf[QT][D / 32];
    WaveAcc<D> acc[QT];
#pragma unroll
    for (int c = 0; c < QT; ++c) {
        const int32_t col = kTile * c + r < nq_w ? kTile * c + r : nq_w - 1;   // padding columns shadow the last query
        pq[c] = pos0_w + col;
        if (computes) {
            const uint4* qrow = q16 + ((int64_t)(tq0_w + col) * prm.Hq + (int64_t)h * prm.G + head) * (D / 8) + q;
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) qf[c][kk] = as_bf16x8(qrow[kk * 4]);
        }
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) acc[c].o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        acc[c].m = -INFINITY;
        acc[c].l = 0.f;
    }

    // A ring of kTiles LDS tiles: while step s is computed the copies of steps s + 1 .. s + kAhead
    // are in flight (one step ahead is not enough: a copy takes longer than a step's arithmetic).
    // Copies are issued for steps past the last one too (clamped to it), so that every wave always
    // has the same number in flight and one wait count fits all.  The tiles are separate arrays
    // and the loop is unrolled over them, so that each LDS access names its array: the compiler
    // then orders an LDS read only after the copies into the same tile, not after all of them.
    const int32_t last_t0 = (n_steps - 1) * kStep;
    auto tile = [&](auto I) -> uint4* {
        if constexpr (decltype(I)::value == 0) return tile0;
        else if constexpr (decltype(I)::value == 1) return tile1;
        else if constexpr (decltype(I)::value == 2) return tile2;
        else return tile3;
    };
    auto pages_of = [&](int32_t t0) {
        return step_page_ids(pt_row, min(t0, last_t0), prm.log2P, prm.max_pages, prm.num_pages);
    };
    CopySrc<D> cs;   // set where a loop in which all waves copy begins (not kept through the other loops)
    const int64_t page_stride = ((int64_t)prm.Hs * D) << (prm.log2P - 3);
    auto copy_to = [&](auto I, int32_t t0, StepPages pg) {
        copy_step<D>(tile(I), cs, pg, min(t0, last_t0), prm.log2P, page_stride);
    };
    StepPages pg_next;   // page ids of the next copy, fetched one step early: the copy never waits for them
    StepData<D> sd;   // K of the step about to be computed is read one step early (see below)
    auto read_k = [&](auto I) {
        const uint4* kt = tile(I);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) sd.k[tt][kk] = kt[(4 * kk + q) * 32 + 16 * tt + r];
    };
    // One step.  V of step s from tile I into registers (K is there already), start the copy of
    // step s + kAhead into the tile that step s - 1 used (every wave has passed the barrier
    // since), scores; the K registers are free now and take K of step s + 1 from the next tile
    // while softmax and PV run (all waves would otherwise read LDS at the same moment after every
    // barrier, with the matrix cores idle); then wait until this wave's copies of steps s + 1 and
    // s + 2 have landed and meet the other waves.
    auto step = [&](auto I, int32_t s) {
        constexpr int kI = decltype(I)::value;
        const int32_t t0 = s * kStep;
        if (computes) {
            const uint4* vt = tile(I) + (D / 8) * 32;
#pragma unroll
            for (int nt = 0; nt < D / 16; ++nt) sd.v[nt] = vt[q * D + 16 * nt + r];
        }
        copy_to(std::integral_constant<int, (kI + kAhead) % kTiles>{}, t0 + kAhead * kStep, pg_next);
        pg_next = pages_of(t0 + (kAhead + 1) * kStep);
        if (computes) {
            if (t0 + kStep > kv_end) mask_v_tail<D>(sd, kv_end - (t0 + 8 * q));
            // Scores of all column tiles first, then softmax and PV tile by tile: the vector work
            // of one tile's softmax then runs while the matrix cores finish the other tile's
            // products.
            float sv[QT][8];
#pragma unroll
            for (int c = 0; c < QT; ++c) qk_scores<D>(qf[c], sd, sv[c]);
            read_k(std::integral_constant<int, (kI + 1) % kTiles>{});
            if (t0 + kStep - 1 > pos0_w) {   // the step reaches past the first query's position: causal mask
                const int32_t first = t0 + 8 * q;
#pragma unroll
                for (int c = 0; c < QT; ++c)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (first + j > pq[c]) sv[c][j] = -INFINITY;
            }
            // The softmax of all column tiles as one stretch of straight-line code (independent
            // dependency chains for the scheduler to interleave), one test for the rare rescale,
            // then all PV products.  Token 0 is visible to every column, so the max is finite.
            StepProbs pr[QT];
#pragma unroll
            for (int c = 0; c < QT; ++c) pr[c] = softmax_probs_lazy<D, F32OUT>(sv[c], prm.scale_log2e, acc[c]);
#pragma unroll
            for (int c = 0; c < QT; ++c) pv_accumulate<D, F32OUT>(sd, pr[c], acc[c]);
        }
        copies_landed_but<D, kAhead - 2>();   // steps s + 1 and s + 2 have landed
        __builtin_amdgcn_s_barrier();
    };

    // The same work as a three-stage pipeline (workgroups of 8 waves, which have the registers for
    // it).  A wave issues an instruction every five or six cycles at best, a matrix instruction
    // keeps the matrix core busy for sixteen or more, and vector instructions that do not depend
    // on it run in its shadow: so the step's three parts must not follow each other (scores,
    // then softmax, then PV: the matrix cores idle during the softmax and the vector units
    // during the products) but run side by side on different steps.  Iteration s holds, in one
    // stretch of straight-line code with no dependencies between the three: the PV products of
    // step s - 1 (probabilities and V from the previous iteration), the exponentials, sums and
    // packing of step s (its scores came out of the previous iteration), and the score products
    // of step s + 1 (K read at the start of the iteration).  Iteration 0 multiplies zero
    // probabilities, the last one scores the ring's clamped copy of the last step and drops them.
    // What has to branch comes before that stretch: the causal mask of the steps on the diagonal
    // and the (rare) move of the softmax reference, which first completes the pending PV products
    // because their probabilities are relative to the old reference.
    StepProbs pr[QT];
    float sv[QT][8];
    // K of step s + 1 is asked for at the start of the iteration; the stretch itself is fenced into
    // three parts so that the LDS reads stay where their latency is covered: PV products with the
    // exponents, exponentials, packing and sums, then the reads of V (into the registers the PV
    // products have just read), then the score products; V arrives during the score products,
    // before the barrier's wait.
    uint4 k_next[2][D / 32];
    auto ask_k = [&](auto I) {
        constexpr int kI = decltype(I)::value;
        const uint4* kt = tile(std::integral_constant<int, (kI + 1) % kTiles>{});
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) k_next[tt][kk] = kt[(4 * kk + q) * 32 + 16 * tt + r];
    };
    // Sum of a step's probabilities of one column in this lane.  For a bf16 result it is the sum
    // of the ROUNDED probabilities, the ones the PV products use (numerator and denominator of
    // the softmax then carry the same rounding), taken two at a time by the bf16 dot product.
    auto step_sum = [&](const float (&p)[8], const StepProbs& now) -> float {
        if constexpr (F32OUT) {
            return ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        } else {
            const uint4 w = __builtin_bit_cast(uint4, now.hi);
            const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
            float acc2 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), ones, 0.f, false);
            acc2 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), ones, acc2, false);
            acc2 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), ones, acc2, false);
            return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), ones, acc2, false);
        }
    };
    // The reference of a column is NOT moved in this loop.  It is the exact maximum of the column's
    // scores in step 0; a later score above it only makes probabilities larger than 1, which
    // neither bf16 (a relative rounding) nor the fp32 sums mind, and the final division makes
    // the result the same.  Moving it would take a test of the step's scores and a branch in
    // every step, and a branch on a vector result waits until the wave's matrix instructions in
    // flight have finished: a quarter of the step's time.  What can go wrong without it is
    // overflow when scores rise by tens of powers of two above those of the first 32 tokens;
    // that shows in the row sums, which are tested once after the loop (kSumLimit), and such a
    // workgroup runs its block again through the exact loop below.
    auto products = [&](auto I, int32_t s) {
        const int32_t t0 = s * kStep;
        if (t0 + kStep - 1 > pos0_w) {   // the step reaches past the first query's position: causal mask
            const int32_t first = t0 + 8 * q;
#pragma unroll
            for (int c = 0; c < QT; ++c)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (first + j > pq[c]) sv[c][j] = -INFINITY;
        }
        float t[QT][8], p[QT][8], sum[QT];
        StepProbs now[QT];
#pragma unroll
        for (int c = 0; c < QT; ++c) pv_accumulate<D, F32OUT>(sd, pr[c], acc[c]);
#pragma unroll
        for (int c = 0; c < QT; ++c) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                t[c][j] = fmaf(sv[c][j], prm.scale_log2e, -acc[c].m);
                p[c][j] = __builtin_amdgcn_exp2f(t[c][j]);
            }
        }
#pragma unroll
        for (int i = 0; i < QT * 8; ++i) {   // one product, one exponent, one exponential, ..
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // K has had the PV products to arrive: saying so here keeps the wait for it from also
        // covering the reads of V that follow.
        __builtin_amdgcn_s_waitcnt((7 << 4) | 0xF | (3 << 14));
        const uint4* vt = tile(I) + (D / 8) * 32;
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) sd.v[nt] = vt[q * D + 16 * nt + r];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < QT; ++c) qk_scores_of<D>(qf[c], k_next, sv[c]);
#pragma unroll
        for (int c = 0; c < QT; ++c) {   // packing and sums in the shadow of the score products
            now[c] = pack_probs<F32OUT>(p[c]);
            sum[c] = step_sum(p[c], now[c]);
        }
#pragma unroll
        for (int i = 0; i < QT * 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x002, 1, 1);
        }
#pragma unroll
        for (int c = 0; c < QT; ++c) {
            acc[c].l += sum[c];
            pr[c] = now[c];
        }
    };
    auto feed = [&](auto I, int32_t s) {   // the copy of step s + kAhead, the page ids of the one after
        constexpr int kI = decltype(I)::value;
        copy_to(std::integral_constant<int, (kI + kAhead) % kTiles>{}, (s + kAhead) * kStep, pg_next);
        pg_next = pages_of((s + kAhead + 1) * kStep);
    };
    // Who copies.  A wave issues an instruction every eight cycles or so whatever its kind, and two
    // waves per SIMD do not fill the SIMD's issue port: what a computing wave does not have to
    // issue is time won.  With fewer than 8 units the workgroup has waves that compute nothing;
    // the last 1, 2 or 4 of them then do all the copying (16, 8 or 4 pieces per lane and step
    // for head_dim 128) and fetch the page ids, and the computing waves issue nothing but their
    // products, the softmax and their LDS reads.  With 8 units all waves copy, two pieces per
    // lane.
    // (An fp32 result splits every probability into two bf16 parts: half again as many PV products
    // and not enough registers for three steps side by side; it keeps the exact loop below.)
    constexpr bool kPipelined = !F32OUT;
    const int32_t n_cp = !kPipelined ? 0 : prm.U <= 4 ? 4 : prm.U <= 6 ? 2 : prm.U == 7 ? 1 : 0;
    const int32_t first_cp = 8 - n_cp;

    const bool shared_copy = n_cp == 0;
    auto iter = [&](auto I, int32_t s) {
        // (nothing is outstanding here; said explicitly, it keeps the first wait of the stretch,
        // the one for V of the previous step, from covering the reads of K asked for now)
        __builtin_amdgcn_s_waitcnt((7 << 4) | 0xF | (3 << 14));
        if (computes) ask_k(I);
        if (shared_copy) feed(I, s);
        if (computes) products(I, s);
        if (shared_copy) copies_landed_but<D, kAhead - 2>();
        else __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (0xF) | (3 << 14));   // LDS reads returned (vmcnt untouched)
        __builtin_amdgcn_s_barrier();
    };

    if constexpr (kPipelined) {
        if (n_cp > 0 && wave >= first_cp) {
            // ---- a copying wave (page size and number of copying waves as compile-time constants,
            // so that everything about a piece but its page is an immediate)
            const int32_t cw = wave - first_cp;
#define ROLL_COPIER(LOG2P, NCP)                                                                                     \
    copier_loop<D, LOG2P, NCP>(tile0, tile1, tile2, tile3, k_pages, v_pages, pt_row, h, cw, lane, n_steps, page_stride, \
                               prm.max_pages, prm.num_pages)
            if (prm.log2P == 4) {
                if (n_cp == 1) ROLL_COPIER(4, 1); else if (n_cp == 2) ROLL_COPIER(4, 2); else ROLL_COPIER(4, 4);
            } else if (prm.log2P == 5) {
                if (n_cp == 1) ROLL_COPIER(5, 1); else if (n_cp == 2) ROLL_COPIER(5, 2); else ROLL_COPIER(5, 4);
            } else {
                if (n_cp == 1) ROLL_COPIER(6, 1); else if (n_cp == 2) ROLL_COPIER(6, 2); else ROLL_COPIER(6, 4);
            }
#undef ROLL_COPIER
        } else if (n_cp > 0 && !computes) {   // a wave with nothing to do keeps the barriers company
            for (int32_t s = 0; s <= n_steps; ++s) __builtin_amdgcn_s_barrier();
        } else {
            if (shared_copy) {
                cs = copy_sources<D>(k_pages, v_pages, h, prm.log2P);
                copy_to(std::integral_constant<int, 0>{}, 0, pages_of(0));
                copy_to(std::integral_constant<int, 1>{}, kStep, pages_of(kStep));
                copy_to(std::integral_constant<int, 2>{}, 2 * kStep, pages_of(2 * kStep));
                pg_next = pages_of(kAhead * kStep);
                copies_landed_but<D, kAhead - 2>();
            }
            __builtin_amdgcn_s_barrier();
            if (computes) {
                read_k(std::integral_constant<int, 0>{});
#pragma unroll
                for (int c = 0; c < QT; ++c) {
                    qk_scores<D>(qf[c], sd, sv[c]);
                    pr[c].hi = as_bf16x8(make_uint4(0u, 0u, 0u, 0u));
                    pr[c].lo = pr[c].hi;
                }
#pragma unroll
                for (int nt = 0; nt < D / 16; ++nt) sd.v[nt] = make_uint4(0u, 0u, 0u, 0u);
                // The reference of a column: the exact maximum of its scores in step 0 (token 0 is
                // visible to every column, so it is finite).
                float s0[QT][8];
#pragma unroll
                for (int c = 0; c < QT; ++c)
#pragma unroll
                    for (int j = 0; j < 8; ++j) s0[c][j] = 8 * q + j > pq[c] ? -INFINITY : sv[c][j];
#pragma unroll
                for (int c = 0; c < QT; ++c) move_reference<D>(s0[c], prm.scale_log2e, acc[c]);
            }
            ROLL_PF_STAMP(tl_loop);
            for (int32_t s = 0; s < n_steps; s += kTiles) {   // n_steps is the same for the whole workgroup
                iter(std::integral_constant<int, 0>{}, s);
                if (s + 1 < n_steps) iter(std::integral_constant<int, 1>{}, s + 1);
                if (s + 2 < n_steps) iter(std::integral_constant<int, 2>{}, s + 2);
                if (s + 3 < n_steps) iter(std::integral_constant<int, 3>{}, s + 3);
            }
            ROLL_PF_STAMP(tl_done);
            if (computes) {   // the PV products of the last step, whose tokens past the end count for nothing
                if (n_steps * kStep > kv_end) mask_v_tail<D>(sd, kv_end - ((n_steps - 1) * kStep + 8 * q));
                bool suspect = false;
#pragma unroll
                for (int c = 0; c < QT; ++c) {
                    pv_accumulate<D, F32OUT>(sd, pr[c], acc[c]);
                    suspect |= !(acc[c].l < kSumLimit);
                }
                if (suspect) s_redo = 1;
            }
        }
        // Every copy of the loop above must have landed before the tiles may be used again.
        __builtin_amdgcn_s_waitcnt((7 << 4) | (0xF << 8));
        __syncthreads();
        if (s_redo == 0) {
            if (!computes) return;
#pragma unroll
            for (int c = 0; c < QT; ++c) {
                acc[c].l = sum_over_q(acc[c].l);
                if (kTile * c + r < nq_w) {
                    const int64_t idx = ((int64_t)(tq0_w + kTile * c + r) * prm.Hq + (int64_t)h * prm.G + head) * D + 4 * q;
                    store_result<D>(acc[c], out, idx, F32OUT);
                }
            }
#ifdef ROLL_ATTN_TIMELINE
            if (wave == 0 && lane == 0 && g_pf_timeline != nullptr && blockIdx.x < g_pf_timeline_blocks) {
                uint32_t hw, xcc;
                asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
                asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
                uint64_t* o = g_pf_timeline + 8 * (size_t)blockIdx.x;
                o[0] = tl_entry;
                o[1] = tl_found;
                o[2] = tl_loop;
                o[3] = tl_done;
                o[4] = wall_clock64();
                o[5] = ((uint64_t)(xcc & 0xF) << 32) | hw;
                o[6] = (uint64_t)n_steps;
                o[7] = 1;
            }
#endif
            return;
        }
#pragma unroll
        for (int c = 0; c < QT; ++c) {
#pragma unroll
            for (int nt = 0; nt < D / 16; ++nt) acc[c].o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            acc[c].m = -INFINITY;
            acc[c].l = 0.f;
        }
    }

    // ---- the exact loop: all of the first 8 waves copy, the reference moves whenever a step's
    // scores rise above it.
    cs = copy_sources<D>(k_pages, v_pages, h, prm.log2P);
    copy_to(std::integral_constant<int, 0>{}, 0, pages_of(0));
    copy_to(std::integral_constant<int, 1>{}, kStep, pages_of(kStep));
    copy_to(std::integral_constant<int, 2>{}, 2 * kStep, pages_of(2 * kStep));
    pg_next = pages_of(kAhead * kStep);
    copies_landed_but<D, kAhead - 2>();
    __builtin_amdgcn_s_barrier();
    if (computes) read_k(std::integral_constant<int, 0>{});
    for (int32_t s = 0; s < n_steps; s += kTiles) {
        step(std::integral_constant<int, 0>{}, s);
        if (s + 1 < n_steps) step(std::integral_constant<int, 1>{}, s + 1);
        if (s + 2 < n_steps) step(std::integral_constant<int, 2>{}, s + 2);
        if (s + 3 < n_steps) step(std::integral_constant<int, 3>{}, s + 3);
    }

    if (!computes) return;
#pragma unroll
    for (int c = 0; c < QT; ++c) {
        acc[c].l = sum_over_q(acc[c].l);
        if (kTile * c + r < nq_w) {
            const int64_t idx = ((int64_t)(tq0_w + kTile * c + r) * prm.Hq + (int64_t)h * prm.G + head) * D + 4 * q;
            store_result<D>(acc[c], out, idx, F32OUT);
        }
    }
}

// Profiling events of the calling thread (roll_prof_prefill_events).
thread_local hipEvent_t t_ev_begin = nullptr, t_ev_end = nullptr;
// Units per workgroup of the calling thread's launches, 0 = chosen per launch (roll_prof_prefill_units).
thread_local int32_t t_units = 0;

int validate(const roll_prefill_desc* d) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->num_chunks < 0 || d->num_tokens < 0) return roll::fail(ROLL_ERR_INVALID_ARG, "num_chunks and num_tokens must be >= 0");
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads != 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "num_q_heads must be a positive multiple of num_kv_heads");
    if (d->head_dim != 64 && d->head_dim != 128) return roll::fail(ROLL_ERR_INVALID_ARG, "head_dim must be 64 or 128");
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64");
    if (d->max_pages_per_seq <= 0 || d->num_pages <= 0 || d->num_slots <= 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq, num_pages and num_slots must be > 0");
    if ((int64_t)d->max_pages_per_seq * d->page_size > (1 << 24))
        return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq * page_size above 2^24 tokens");
    if ((int64_t)d->num_pages * d->page_size > INT32_MAX) return roll::fail(ROLL_ERR_INVALID_ARG, "pool above 2^31 tokens");
    if ((int64_t)d->num_tokens * d->num_q_heads * d->head_dim > ((int64_t)1 << 40))
        return roll::fail(ROLL_ERR_INVALID_ARG, "num_tokens too large");
    if (d->out_dtype != ROLL_BF16 && d->out_dtype != ROLL_F32) return roll::fail(ROLL_ERR_INVALID_ARG, "out_dtype must be ROLL_BF16 or ROLL_F32");
    if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return roll::fail(ROLL_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    return ROLL_OK;
}

}  // namespace

extern "C" int roll_prefill_attn(const void* q, const void* k_new, const void* v_new, const int32_t* chunk_slot,
                                 const int32_t* chunk_start, const int32_t* chunk_offset, void* k_pages,
                                 void* v_pages, const int32_t* page_table, void* out, const roll_prefill_desc* d,
                                 void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    if (d->num_chunks == 0 || d->num_tokens == 0) return ROLL_OK;
    if (!q || !k_new || !v_new || !chunk_slot || !chunk_start || !chunk_offset || !k_pages || !v_pages || !page_table || !out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(q, 16) || !roll::aligned(k_new, 16) || !roll::aligned(v_new, 16) || !roll::aligned(k_pages, 16) ||
        !roll::aligned(v_pages, 16) || !roll::aligned(out, 16))
        return roll::fail(ROLL_ERR_INVALID_ARG, "q, k_new, v_new, k_pages, v_pages, out must be 16-byte aligned");
    hipStream_t stream = (hipStream_t)stream_v;
    PrefillParams prm{};
    prm.C = d->num_chunks;
    prm.T = d->num_tokens;
    prm.Hq = d->num_q_heads;
    prm.Hkv = d->num_kv_heads;
    prm.Hs = roll::page_stride_heads(d->page_stride, d->num_kv_heads, d->page_size, d->head_dim);
    if (prm.Hs == 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_stride must be 0 or a multiple of page_size * head_dim that holds all KV heads");
    prm.G = d->num_q_heads / d->num_kv_heads;
    prm.log2P = d->page_size == 16 ? 4 : (d->page_size == 32 ? 5 : 6);
    prm.max_pages = d->max_pages_per_seq;
    prm.num_pages = d->num_pages;
    prm.num_slots = d->num_slots;
    prm.out_f32 = d->out_dtype == ROLL_F32;
    const float scale = d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / sqrtf((float)d->head_dim);
    prm.scale_log2e = scale * 1.44269504088896340736f;

    const int64_t k_items = (((int64_t)prm.T + 15) / 16 * 16) * prm.Hkv * (d->head_dim / 8);   // tokens in sixteens
    const int64_t k_blocks = (k_items + 255) / 256;
    // at most T / 8 + 2 C octets of positions (a chunk may begin and end inside one); one wave per
    // octet, KV head and 64 head-dim elements, four waves per workgroup
    const int64_t v_waves = (((int64_t)prm.T + 7) / 8 + 2 * (int64_t)prm.C) * prm.Hkv * (d->head_dim / 64);
    const int64_t v_blocks = (v_waves + 3) / 4;
    if (k_blocks + v_blocks > INT32_MAX) return roll::fail(ROLL_ERR_INVALID_ARG, "too many tokens");
    append_chunks<<<(unsigned)(k_blocks + v_blocks), 256, 0, stream>>>(
        (const uint4*)k_new, (const uint16_t*)v_new, chunk_slot, chunk_start, chunk_offset, (uint4*)k_pages,
        (uint4*)v_pages, page_table, prm, d->head_dim, (int32_t)k_blocks);
    ROLL_HIP_CHECK(hipGetLastError());

    constexpr int qt = 2;   // column tiles (16 query tokens) per wave
    // How many units (span of query tokens x query head) a workgroup takes, one per computing wave.
    // A compute unit holds one workgroup of 8 waves; what it gets done depends on how many of
    // them compute (measured on 8 x 4096 tokens with 1 .. 8 query heads per KV head and one span
    // per workgroup, relative to one wave; 7 waves and a copying one beat 8 that share the
    // copying).  The number is the one for which (workgroups, at most one per compute unit) x
    // (that yield) is largest: a small launch is better off with more, lighter workgroups.
    const int span = kTile * qt;
    const int64_t spans_bound = ((int64_t)prm.T + span - 1) / span + prm.C;   // each chunk ends with at most one partial span
    auto workgroups = [&](int units) { return ((spans_bound * prm.G + units - 1) / units + prm.C) * prm.Hkv; };
    static const double kYieldPipelined[9] = {0.0, 1.0, 2.0, 2.63, 3.4, 3.54, 4.18, 4.6, 4.44};
    prm.U = 1;
    if (t_units >= 1) {
        prm.U = t_units;
    } else {
        double best = 0.0;
        for (int units = 1; units <= kCopyWaves; ++units) {
            const int64_t wgs = workgroups(units);
            const double yield = prm.out_f32 ? (units <= 4 ? (double)units : 4.0 + 0.15 * (units - 4)) : kYieldPipelined[units];
            const double score = (double)(wgs < kComputeUnits ? wgs : kComputeUnits) * yield;
            if (score > best) {
                best = score;
                prm.U = units;
            }
        }
    }
    // At most this many workgroups: every chunk's last one may be partly empty.
    const int64_t grid = workgroups(prm.U);
    if (grid > INT32_MAX) return roll::fail(ROLL_ERR_INVALID_ARG, "too many query blocks");
    const int threads = kCopyThreads;   // 8 waves
    if (t_ev_begin) ROLL_HIP_CHECK(hipEventRecord(t_ev_begin, stream));
#define ROLL_LAUNCH_PREFILL(DIM, F32)                                                                         \
    prefill_attn<DIM, qt, F32><<<(unsigned)grid, threads, 0, stream>>>(                                       \
        (const uint4*)q, (const uint4*)k_pages, (const uint4*)v_pages, page_table, chunk_slot, chunk_start,    \
        chunk_offset, out, prm)
    if (d->head_dim == 128) {
        if (prm.out_f32) ROLL_LAUNCH_PREFILL(128, true); else ROLL_LAUNCH_PREFILL(128, false);
    } else {
        if (prm.out_f32) ROLL_LAUNCH_PREFILL(64, true); else ROLL_LAUNCH_PREFILL(64, false);
    }
#undef ROLL_LAUNCH_PREFILL
    ROLL_HIP_CHECK(hipGetLastError());
    if (t_ev_end) ROLL_HIP_CHECK(hipEventRecord(t_ev_end, stream));
    return ROLL_OK;
}

extern "C" int roll_prof_prefill_timeline(void* buffer, size_t buffer_bytes) {
#ifdef ROLL_ATTN_TIMELINE
    uint64_t* p = (uint64_t*)buffer;
    const size_t blocks = buffer ? buffer_bytes / (8 * sizeof(uint64_t)) : 0;
    const uint32_t n = blocks > UINT32_MAX ? UINT32_MAX : (uint32_t)blocks;
    if (buffer && !roll::aligned(buffer, 8)) return roll::fail(ROLL_ERR_INVALID_ARG, "timeline buffer must be 8-byte aligned");
    ROLL_HIP_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(g_pf_timeline_blocks), &n, sizeof n));
    ROLL_HIP_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(g_pf_timeline), &p, sizeof p));
    return ROLL_OK;
#else
    (void)buffer;
    (void)buffer_bytes;
    return roll::fail(ROLL_ERR_INVALID_ARG, "this library was built without ROLL_ATTN_TIMELINE "
                                            "(python -m paper_2510_11345_amd.build --timeline builds one with it)");
#endif
}

extern "C" int roll_prof_prefill_units(int32_t units) {
    if (units < 0 || units > 8) return roll::fail(ROLL_ERR_INVALID_ARG, "units must be 0 (chosen per launch) or 1 .. 8");
    t_units = units;
    return ROLL_OK;
}

extern "C" int roll_prof_prefill_events(void* begin, void* end) {
    if ((begin == nullptr) != (end == nullptr)) return roll::fail(ROLL_ERR_INVALID_ARG, "begin and end must both be set or both NULL");
    t_ev_begin = (hipEvent_t)begin;
    t_ev_end = (hipEvent_t)end;
    return ROLL_OK;
}
