// How decode attention deals the rows of a batch to its persistent workgroups: shared by the
// kernel (rows' prefix sums in LDS) and by roll_decode_attn_ranges on the host (the same sums
// in host memory), so that what the host reports is what the kernel does.
//
// ROLL Flash (arXiv 2510.11345) Section 1: response lengths are long-tailed, so the rows of a
// decode batch differ in length by orders of magnitude and have to be cut to share the chip.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace roll {
namespace attn {

constexpr int kDealStep = 32;      // tokens per step (the unit of work)
constexpr int kGroupWaves = 4;     // wavefronts per workgroup
constexpr int kMinSteps = 4;       // do not cut a small batch into ranges shorter than this
constexpr int kMaxSlots = 32768;   // piece slots: two per (range of row steps, KV head)

// Ranges of row steps a launch of `waves` persistent waves can use (before the limits that depend
// on the batch): one per workgroup, times the cut within a workgroup when there are fewer KV
// heads than waves; never more than the piece slots allow.
__host__ __device__ inline int32_t ranges_cut(int32_t Hkv) {
    return (Hkv < kGroupWaves && kGroupWaves % Hkv == 0) ? kGroupWaves / Hkv : 1;
}
__host__ __device__ inline int32_t max_ranges(int32_t waves, int32_t Hkv) {
    const int32_t by_waves = waves / kGroupWaves * ranges_cut(Hkv);
    const int32_t by_slots = kMaxSlots / (2 * Hkv);
    const int32_t n = by_waves < by_slots ? by_waves : by_slots;
    return n < 1 ? 1 : n;
}

// How the row steps are cut into ranges.  A wave runs alone on its SIMD, so what a stream costs
// beyond its steps (the merge or the result store of the one before, its Q, its first page ids and
// first K/V bytes, each a round trip to memory with nothing to hide behind) is time in which the
// wave streams nothing: about one step, measured.  Ranges are therefore equal in
// cost, not in steps: on a line where every row that holds tokens takes kRowCost units followed
// by kStepCost units for each of its steps, range c begins at position floor(c T / NC) of the T
// units in all, and owns the steps that begin at or after that position and before the next
// range's.  A range with many short rows gets fewer steps.
constexpr int32_t kStepCost = 2;
constexpr int32_t kRowCost = 2;
struct Deal {
    int64_t T;   // total cost units over all rows (one KV head)
    int32_t NC;  // ranges in use
    __host__ __device__ Deal(int32_t steps, int32_t rows, int32_t waves, int32_t Hkv)
        : T((int64_t)steps * kStepCost + (int64_t)rows * kRowCost) {
        const int32_t want = (steps + kMinSteps - 1) / kMinSteps;
        const int32_t most = max_ranges(waves, Hkv);
        NC = want < 1 ? 1 : (want < most ? want : most);
    }
    __host__ __device__ int64_t boundary(int32_t c) const { return (int64_t)c * T / NC; }
    // the range that owns a step whose first cost unit is x: the last c with boundary(c) <= x
    __host__ __device__ int32_t owner(int64_t x) const { return (int32_t)(((x + 1) * NC + T - 1) / T - 1); }
    // the slots of (range c, KV head h): 0 for a piece that begins the range, 1 for one that ends it
    __host__ __device__ int64_t slot(int32_t c, int32_t h, int32_t Hkv, bool begins) const {
        return ((int64_t)c * Hkv + h) * 2 + (begins ? 0 : 1);
    }
};

// pre[b] = steps of the rows before b (B + 1 entries), live[b] = rows with tokens before b.
// Position of row b on the cost line.
__host__ __device__ inline int64_t cost_pre(const int32_t* pre, const uint16_t* live, int32_t b) {
    return (int64_t)pre[b] * kStepCost + (int64_t)live[b] * kRowCost;
}

// The first step of the range whose boundary is position x of the cost line, given the row `lo`
// that holds x: the last row with cost_pre(lo) <= x (it has tokens).
__host__ __device__ inline int32_t first_step_in_row(int64_t x, int32_t lo, const int32_t* pre, const uint16_t* live) {
    const int64_t local = x - cost_pre(pre, live, lo);
    const int32_t n = pre[lo + 1] - pre[lo];
    const int64_t k = local <= kRowCost ? 0 : (local - kRowCost + kStepCost - 1) / kStepCost;
    return pre[lo] + (int32_t)(k < n ? k : n);
}

// The first step range `range` owns (the total number of steps for range >= NC).
__host__ __device__ inline int32_t first_step(const Deal& deal, int32_t range, int32_t B, const int32_t* pre,
                                              const uint16_t* live) {
    if (range >= deal.NC) return pre[B];
    const int64_t x = deal.boundary(range);
    int32_t lo = 0, hi = B;  // invariant: cost_pre(lo) <= x < cost_pre(hi); row lo ends up with tokens
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (cost_pre(pre, live, mid) <= x) lo = mid; else hi = mid;
    }
    return first_step_in_row(x, lo, pre, live);
}

}  // namespace attn
}  // namespace roll
