// Temperature / top-p sampling with log-prob recording for gfx950.
//
// ROLL Flash (arXiv 2510.11345) Appendix A.1: rollout samples with a given
// temperature and top_p (top_k off, one beam) and the engine's probability of
// the sampled token is the denominator of the truncated importance weight, so
// the step must return, next to each token, its log-prob under the
// distribution it was actually drawn from.
//
// One workgroup of 1024 threads per row.
//   top_p == 1: ONE sweep over the row computes the online (max, sum-exp) for
//     the log-sum-exp and runs the Gumbel-max race.
//   top_p <  1: sweep 1 finds max z.  Sweep 2 finds the upper 16 bits of the
//     order-preserving integer key of the cut value x_cut: a histogram in LDS
//     over the 16-bit key prefixes of a window of four top-byte values at and
//     below the row max's, entries below the window going to bins by top byte;
//     every entry adds exp(z - max) in 2^-40 fixed point (integer adds commute,
//     so the cut does not depend on thread timing), and a block-wide scan in
//     descending key order picks the range at which the running mass reaches
//     ceil(top_p * total).  A cut below the window takes one more sweep (the
//     second key byte), fp32 logits two more (the lower 16 key bits).  The last
//     sweep runs the race over logits >= x_cut, drawing random numbers only
//     for the Philox blocks that hold a kept entry (gathered by wave in LDS).
//
// The Gumbel-max race is exact and cheap.  With g(u) = -log(-log u) and
// -log u >= 1 - u, an entry can only win if  1 - u <= exp(z - best), best being
// any lower bound of the row's best perturbed logit.  exp(z - ref) is needed
// for the log-sum-exp anyway, so the test costs a convert, a fused multiply-add
// and a compare per entry on top of the Philox draw (and most vectors are
// dismissed by one test of their largest word against their largest
// exponential); the few entries that pass are evaluated in fp64 (division by
// the temperature and both logs), the arithmetic the definition is stated in.
// The first bound comes from an fp32 lower bound of the first vector's
// entries; a bound that moves is shared by the row's 16 waves through LDS.
// The integer multiplies of Philox are the bulk of the arithmetic: each round
// is two 32x32->64 products (v_mad_u64_u32) and two three-input xors.
#include <cfloat>
#include <cmath>
#include <type_traits>

#include "common.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWavesPerBlock = kThreads / 64;
constexpr int kRadixBits = 8;              // one byte of the key per radix level
constexpr int kBins = 1 << kRadixBits;
constexpr int kCopies = 16;                // copies of every bin, picked by lane % 16, so that lanes
                                           // adding to one hot bin land on different LDS banks
constexpr double kLog2ed = 1.44269504088896340736;
constexpr float kLog2e = 1.44269504088896340736f;

struct SampleParams {
    int32_t V;
    int64_t row_stride;
    float k2;  // log2(e) / temperature: z in log2 units is x * k2
    double temperature;
    float top_p;
    uint32_t seed_lo, seed_hi, step_lo, step_hi;
    int32_t policy_version;
    int32_t* policy_version_out;  // [B] or NULL: the version tag recorded beside every log-prob
};

// ---- Philox4x32-10 (Salmon et al., SC'11) ----------------------------------
struct Philox4 { uint32_t w[4]; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        // a ^ b ^ c in one instruction (v_bitop3_b32, truth table 0x96)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96);
        c0 = n0; c1 = (uint32_t)pb; c2 = n2; c3 = (uint32_t)pa;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// ---- element access ---------------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<uint16_t> {  // bf16 bit patterns
    static constexpr int kVec = 8;
    static constexpr int kKeyBits = 16;
    __device__ static uint4 minus_inf_vector() { return make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u); }
    __device__ static float widen(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
    __device__ static void unpack(const uint4& v, float (&x)[8]) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[2 * j] = __uint_as_float(w[j] << 16);
            x[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
};
template <> struct Elem<float> {
    static constexpr int kVec = 4;
    static constexpr int kKeyBits = 32;
    __device__ static uint4 minus_inf_vector() { return make_uint4(0xFF800000u, 0xFF800000u, 0xFF800000u, 0xFF800000u); }
    __device__ static float widen(float f) { return f; }
    __device__ static void unpack(const uint4& v, float (&x)[4]) {
        x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y);
        x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
    }
};

// Order-preserving key: larger float <=> larger unsigned key.  Adding +0 turns -0 into +0, so
// that the two zeros, equal as values, are one class of the cut.
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t b = __float_as_uint(x + 0.0f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    const uint32_t b = (k >> 31) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(b);
}

// Calls f.run<N>(i0, x, active) for every aligned vector of the row and f.run<1> for the
// tail.  Every lane of the workgroup makes the same number of calls (inactive ones carry
// active == false and logits of -inf), so the bodies may use wave-wide operations.  The next
// vector is requested before the current one is processed.
template <typename T, typename F>
__device__ __forceinline__ void sweep(const T* __restrict__ row, int32_t V, F& f) {
    constexpr int N = Elem<T>::kVec;
    const int32_t nvec = V / N;
    const uint4* __restrict__ row16 = (const uint4*)row;
    const uint4 zero = Elem<T>::minus_inf_vector();
    int32_t vi = (int32_t)threadIdx.x;
    uint4 cur = vi < nvec ? row16[vi] : zero;
    for (int32_t base = 0; base < nvec; base += kThreads) {
        const int32_t vn = vi + kThreads;
        const uint4 nxt = vn < nvec ? row16[vn] : zero;
        float x[N];
        Elem<T>::unpack(cur, x);
        f.template run<N>(vi * N, x, vi < nvec);
        cur = nxt;
        vi = vn;
    }
    if (nvec * N < V) {
        const int32_t i = nvec * N + (int32_t)threadIdx.x;
        const bool active = i < V;
        float x[1] = {active ? Elem<T>::widen(row[i]) : -INFINITY};
        f.template run<1>(i, x, active);
    }
}

// ---- cross-lane helpers -------------------------------------------------------
__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
    uint64_t b = __builtin_bit_cast(uint64_t, v);
    uint32_t lo = __shfl_xor((uint32_t)b, mask), hi = __shfl_xor((uint32_t)(b >> 32), mask);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask) {
    uint32_t lo = __shfl_xor((uint32_t)v, mask), hi = __shfl_xor((uint32_t)(v >> 32), mask);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int delta) {
    uint32_t lo = __shfl_up((uint32_t)v, delta), hi = __shfl_up((uint32_t)(v >> 32), delta);
    return ((uint64_t)hi << 32) | lo;
}

// ---- sweep bodies -----------------------------------------------------------
template <bool RAW>
struct MaxOnly {  // per-thread max of the raw logits; with RAW also sum exp(x - xm) (online)
    float xm = -FLT_MAX;
    float s_raw = 0.f;
    template <int N> __device__ __forceinline__ void run(int32_t, const float (&x)[N], bool active) {
        if (!active) return;
        float vmax = x[0];
#pragma unroll
        for (int j = 1; j < N; ++j) vmax = fmaxf(vmax, x[j]);
        const float x_new = fmaxf(xm, vmax);
        if (RAW) {
            s_raw *= __builtin_amdgcn_exp2f((xm - x_new) * kLog2e);
#pragma unroll
            for (int j = 0; j < N; ++j) s_raw += __builtin_amdgcn_exp2f((x[j] - x_new) * kLog2e);
        }
        xm = x_new;
    }
};

// The exponentials of a sum are exp2(fma(x, k2, nk)) with nk = -fl(xref k2): relative to
// 2^(-nk) exactly, whatever rounding nk itself carries.  Kept finite so that -inf entries
// give exp2(-inf) = 0 and not inf - inf.
__device__ __forceinline__ float ref_offset(float xref, float k2) { return fminf(-xref * k2, FLT_MAX); }

// Gumbel-max race with the exact filter described at the top of the file.  With LSE the
// per-thread reference logit follows the thread's running max and s accumulates
// sum exp2((x - xref) k2); without it the reference is fixed (the row max) and only the
// race runs.
// CUT: entries below x_cut are not kept (the top-p pass); without it every entry is.
template <bool LSE, bool RAW, bool CUT>
struct Race {
    const SampleParams& p;
    uint32_t row_id;
    float x_cut;             // entries below it are not kept (-inf when top_p == 1)
    float xref;              // reference logit of the exponentials: the running max of this
                             // thread's raw logits (LSE) or the row max (otherwise)
    float s = 0.f;           // sum of exp2((x - xref) k2) over this thread's entries (LSE only)
    float s_raw = 0.f;       // the same at temperature 1 (LSE and RAW only)
    double best = -INFINITY; // best exact perturbed logit of this lane, natural-log units
    int32_t best_i = 0x7FFFFFFF;
    uint32_t* block_thr_key = nullptr;  // LDS: order_key of the largest threshold any wave of the
                                        // workgroup published (set before the first run)
    float thr2 = -INFINITY;  // lower bound of the row's best perturbed logit, log2 units: the largest
                             // exact value this wave has seen, or one another wave published
    uint32_t thr_key = order_key(-INFINITY);
    float nk = 0.f;          // -xref k2 (finite): exponents are formed as fma(x, k2, nk)
    float c = INFINITY;      // 2^32 exp2(-nk - thr2) with a safety factor

    __device__ __forceinline__ void set_ref(float x_new) {
        xref = x_new;
        nk = ref_offset(x_new, p.k2);
    }

    __device__ __forceinline__ void exact(int32_t i, float x, uint32_t word) {
        const double u = ((double)(word >> 9) + 0.5) * 0x1p-23;
        const double y = (double)x / p.temperature - log(-log(u));
        if (y > best || (y == best && i < best_i)) {
            best = y;
            best_i = i;
        }
    }
    __device__ __forceinline__ void share() {
        double b = best;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) b = fmax(b, shfl_xor_f64(b, mask));
        float t = (float)(b * kLog2ed);
        if ((double)t > b * kLog2ed) t = nextafterf(t, -INFINITY);
        publish(nextafterf(t, -INFINITY));
    }
    // t (wave-uniform) bounds the row's best perturbed logit from below, in log2 units: publish
    // it and take what the other waves have published.  Which threshold a wave happens to see
    // only decides how many entries it evaluates exactly, never the result.
    __device__ __forceinline__ void publish(float t) {
        uint32_t k = order_key(t);
        uint32_t seen = 0;
        if ((threadIdx.x & 63) == 0) seen = atomicMax(block_thr_key, k);
        seen = __builtin_amdgcn_readfirstlane(seen);
        k = seen > k ? seen : k;
        if (k > thr_key) {
            thr_key = k;
            thr2 = key_to_float(k);
        }
    }
    __device__ __forceinline__ void refresh_c() { c = __builtin_amdgcn_exp2f(-nk - thr2) * (1.0001f * 0x1p32f); }

    template <int N> __device__ __forceinline__ void run(int32_t i0, const float (&x)[N], bool active) {
        if (CUT) {  // a vector without a kept entry in any lane needs no random numbers
            bool kept = false;
#pragma unroll
            for (int j = 0; j < N; ++j) kept = kept || x[j] >= x_cut;
            if (!__any(kept)) return;
        }
        // requested here, used after the random words are drawn
        const uint32_t block_key = __hip_atomic_load(block_thr_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        uint32_t words[N];
        if (N == 1) {
            const Philox4 r = philox4x32_10((uint32_t)i0 >> 2, row_id, p.step_lo, p.step_hi, p.seed_lo, p.seed_hi);
            words[0] = r.w[i0 & 3];
        } else {
#pragma unroll
            for (int b4 = 0; b4 < N / 4; ++b4) {
                const Philox4 r = philox4x32_10(((uint32_t)i0 >> 2) + b4, row_id, p.step_lo, p.step_hi, p.seed_lo, p.seed_hi);
#pragma unroll
                for (int j = 0; j < 4; ++j) words[4 * b4 + j] = r.w[j];
            }
        }
        (void)active;  // an inactive lane's logits are -inf: they add nothing and cannot pass
        const float (&xa)[N] = x;
        float vmax = xa[0];
        if (LSE) {  // move the reference to the running max when some lane's max grew (rare after
                    // the first vectors; the sums are rescaled only then)
#pragma unroll
            for (int j = 1; j < N; ++j) vmax = fmaxf(vmax, xa[j]);
            if (__any(vmax > xref)) {
                const float x_new = fmaxf(xref, vmax);
                s *= __builtin_amdgcn_exp2f((xref - x_new) * p.k2);
                if (RAW) s_raw *= __builtin_amdgcn_exp2f((xref - x_new) * kLog2e);
                set_ref(x_new);
                refresh_c();
            }
            if (RAW) {
#pragma unroll
                for (int j = 0; j < N; ++j) s_raw += __builtin_amdgcn_exp2f((xa[j] - xref) * kLog2e);
            }
        }
        if (block_key > thr_key) {  // another wave has found a better candidate
            thr_key = block_key;
            thr2 = key_to_float(block_key);
            refresh_c();
        }
        if (__any(thr2 == -INFINITY)) {
            // Nothing bounds the best yet, so every kept entry would pass and be evaluated
            // exactly.  A bound from below in fp32 comes first: -ln u <= (1 - u) / u, so the
            // perturbed logit in log2 units is at least x k2 - log2(1 - u) + log2(u), and both
            // u = (k + 0.5) 2^-23 and 1 - u = (2^23 - 1 - k + 0.5) 2^-23 are exact in fp32 (the
            // 2^-23 cancel).  The margin covers the two hardware logs (1 ulp of a value below 24)
            // and the rounding of k2 and of the product.  The bound is within (1 - u) / 2 of the
            // value itself, so what then passes the test below is little more than the winner.
            float lb = -INFINITY;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const float u_num = (float)(words[j] >> 9) + 0.5f;
                const float one_minus_u_num = (float)((~words[j]) >> 9) + 0.5f;
                const float z2 = x[j] * p.k2;
                const float v = z2 - __builtin_amdgcn_logf(one_minus_u_num) + __builtin_amdgcn_logf(u_num) -
                                (0x1p-16f + fabsf(z2) * 0x1p-21f);
                if (x[j] > -INFINITY && (!CUT || x[j] >= x_cut)) lb = fmaxf(lb, v);
            }
#pragma unroll
            for (int mask = 1; mask < 64; mask <<= 1) lb = fmaxf(lb, __shfl_xor(lb, mask));
            publish(lb);
            refresh_c();
        }
        float e[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            // The exponent keeps full relative accuracy near the reference: the product is not
            // rounded before nk is added.  -inf entries give 0.
            e[j] = __builtin_amdgcn_exp2f(fmaf(xa[j], p.k2, nk));
            if (LSE) s += e[j];
        }
        if (LSE && N > 1) {
            // The vector's largest word against its largest exponential: no entry can pass the
            // test below unless this pair does.
            uint32_t wmax = words[0];
#pragma unroll
            for (int j = 1; j < N; ++j) wmax = wmax > words[j] ? wmax : words[j];
            const float emax = __builtin_amdgcn_exp2f(fmaf(vmax, p.k2, nk));
            if (!__any((float)wmax >= fmaf(-emax, c, 8388606.5f * 512.f))) return;
        }
        bool pass[N];
        bool any_pass = false;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            // With k = word >> 9, 1 - u = (2^23 - 1 - k + 0.5) 2^-23, so 1 - u <= e exp2(..) reads
            // k >= 2^23 - 0.5 - e exp2(..) 2^23.  Both sides are taken times 2^9: the whole word
            // converted to fp32 (rounded to nearest) is at least k 2^9, and the right side is
            // formed one unit of k lower, (2^23 - 1.5) 2^9 - e c (fp32 rounds that by at most a
            // quarter unit), so the test can only let an extra entry through, never hold a winner
            // back.  e = 0 (an entry more than 126 binary orders below a logit of the same row,
            // which the 28 orders a draw can add never make up) with c = inf gives NaN: no pass.
            pass[j] = (float)words[j] >= fmaf(-e[j], c, 8388606.5f * 512.f) && (!CUT || x[j] >= x_cut);
            any_pass = any_pass || pass[j];
        }
        if (__any(any_pass)) {
#pragma unroll
            for (int j = 0; j < N; ++j)
                if (pass[j]) exact(i0 + j, x[j], words[j]);
            share();
            refresh_c();
        }
    }
};

// The race over the kept entries only.  A Philox block serves four consecutive entries, and below
// the cut lies most of the row, so the blocks that hold a kept entry are first gathered, by wave,
// into a queue in LDS (block number and its four logits), and the race runs on 64 gathered blocks
// at a time, one per lane: random numbers are drawn only for blocks that need them.  A wave
// whose first vector has a kept entry in more than half of its blocks (a cut deep in the row)
// skips the queue and races on the vectors as they come.
constexpr int kQueueCap = 128;  // >= 63 left over + 64 pushed; a power of two
constexpr int kQueueBytesPerWave = kQueueCap * (4 * 4 + 4);

template <typename RaceT>
struct CompactRace {
    RaceT& race;
    float* qx;       // [kQueueCap][4] this wave's queue: the logits of a block
    uint32_t* qblk;  // [kQueueCap] and its number (entry index / 4)
    uint32_t head = 0, tail = 0;  // wave-uniform; positions are taken modulo kQueueCap
    int mode = 0;                 // wave-uniform: 0 undecided, 1 through the queue, 2 direct

    __device__ __forceinline__ void drain(uint32_t n) {
        const uint32_t lane = threadIdx.x & 63;
        const uint32_t slot = (tail + lane) & (kQueueCap - 1);
        const bool valid = lane < n;
        __builtin_amdgcn_wave_barrier();
        const float4 v = *(const float4*)(qx + slot * 4);
        const uint32_t blk = qblk[slot];
        __builtin_amdgcn_wave_barrier();
        tail += n;
        const float x4[4] = {valid ? v.x : -INFINITY, valid ? v.y : -INFINITY, valid ? v.z : -INFINITY,
                             valid ? v.w : -INFINITY};
        race.template run<4>((int32_t)((valid ? blk : 0u) * 4u), x4, valid);
    }
    __device__ __forceinline__ void push(uint32_t blk, float x0, float x1, float x2, float x3) {
        const float cut = race.x_cut;
        const bool need = x0 >= cut || x1 >= cut || x2 >= cut || x3 >= cut;
        const unsigned long long mask = __ballot(need);
        if (mask == 0) return;
        const uint32_t pos = head + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                              __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (need) {
            const uint32_t slot = pos & (kQueueCap - 1);
            *(float4*)(qx + slot * 4) = make_float4(x0, x1, x2, x3);
            qblk[slot] = blk;
        }
        head += (uint32_t)__popcll(mask);
        if (head - tail >= 64) drain(64);
    }
    template <int N> __device__ __forceinline__ void run(int32_t i0, const float (&x)[N], bool active) {
        if (N > 1 && mode == 0) {
            const float cut = race.x_cut;
            int needed = 0;
#pragma unroll
            for (int b = 0; b < N / 4; ++b)
                needed += __popcll(__ballot(x[4 * b] >= cut || x[4 * b + 1] >= cut || x[4 * b + 2] >= cut ||
                                            x[4 * b + 3] >= cut));
            mode = needed > 32 * (N / 4) ? 2 : 1;
        }
        if (N > 1 && mode == 2) {
            race.template run<N>(i0, x, active);
            return;
        }
        if (N == 1) {  // the row's tail: one entry of its block per lane
            const int w = i0 & 3;
            push((uint32_t)i0 >> 2, w == 0 ? x[0] : -INFINITY, w == 1 ? x[0] : -INFINITY,
                 w == 2 ? x[0] : -INFINITY, w == 3 ? x[0] : -INFINITY);
        } else {
#pragma unroll
            for (int b = 0; b < N / 4; ++b)
                push(((uint32_t)i0 >> 2) + b, x[4 * b], x[4 * b + 1], x[4 * b + 2], x[4 * b + 3]);
        }
    }
    __device__ __forceinline__ void finish() {
        if (head != tail) drain(head - tail);
    }
};

// w in [0, 1] as 2^-40 fixed point, truncated: the integer and the fractional part of
// w * 2^20 are both exact in fp32, so no 64-bit float conversion is needed.
__device__ __forceinline__ unsigned long long to_fixed40(float w) {
    const float f = w * 0x1p20f;
    const uint32_t a = (uint32_t)f;
    const uint32_t b = (uint32_t)((f - (float)a) * 0x1p20f);
    return ((unsigned long long)a << 20) | b;
}

template <int SHIFT>
struct Histogram {  // adds exp(z - max) in 2^-40 fixed point to the bin of the key's digit
    float k2, nk;   // nk = ref_offset(row max)
    uint32_t prefix;  // the key's bits above SHIFT + kRadixBits must equal this
    unsigned long long* hist;  // [kBins][kCopies]
    uint32_t copy;             // this lane's copy
    // Straight-line code: an entry outside the prefix (or of an inactive lane) adds zero to the
    // bin of its own digit instead of branching around the add; the branches cost more than the
    // adds they saved.
    template <int N> __device__ __forceinline__ void run(int32_t, const float (&x)[N], bool active) {
        unsigned long long fx[N];
        uint32_t slot[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t key = order_key(x[j]);
            bool in = active;
            if (SHIFT + kRadixBits < 32) in = in && (key >> ((SHIFT + kRadixBits) & 31)) == prefix;
            const float w = __builtin_amdgcn_exp2f(fmaf(x[j], k2, nk));
            fx[j] = to_fixed40(in ? w : 0.f);
            slot[j] = ((key >> SHIFT) & (kBins - 1u)) * kCopies + copy;
        }
#pragma unroll
        for (int j = 0; j < N; ++j) atomicAdd(&hist[slot[j]], fx[j]);
    }
};

struct Select {
    uint32_t prefix;            // key bits selected so far (right-aligned)
    unsigned long long above;   // fixed-point mass of keys strictly above the prefix range
    unsigned long long kept;    // above + the mass of the selected range itself
    int32_t found;              // the last selection reached its target
};

// Threads hold the masses of key ranges in descending key order (thread 0 the highest; threads
// with no range pass 0).  Picks the first thread at which above + running sum >= target and
// records its prefix; found stays 0 if the target is not reached.
__device__ void scan_select(unsigned long long mine, uint32_t my_prefix, unsigned long long* s_wave,
                            Select* s_sel, unsigned long long target) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_sel->found = 0;
    unsigned long long incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long v = shfl_up_u64(incl, d);
        if (lane >= d) incl += v;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    unsigned long long base = s_sel->above;
    for (int w = 0; w < wave; ++w) base += s_wave[w];
    incl += base;
    const unsigned long long excl = incl - mine;
    __syncthreads();
    if (excl < target && incl >= target) {
        s_sel->prefix = my_prefix;
        s_sel->above = excl;
        s_sel->kept = incl;
        s_sel->found = 1;
    }
    __syncthreads();
}

// Sum over the workgroup of one value per thread (every thread gets it).
__device__ unsigned long long block_sum_u64(unsigned long long v, unsigned long long* s_wave) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = shfl_up_u64(v, d);
        if (lane >= d) v += o;
    }
    if (lane == 63) s_wave[wave] = v;
    __syncthreads();
    unsigned long long total = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) total += s_wave[w];
    __syncthreads();
    return total;
}

__device__ __forceinline__ unsigned long long top_p_target(float top_p, unsigned long long total) {
    unsigned long long target = (unsigned long long)ceil((double)top_p * (double)total);
    if (target < 1) target = 1;
    if (target > total) target = total;
    return target;
}

// One radix level: histogram of the digit at SHIFT (BITS wide) over the entries whose higher
// key bits equal the prefix chosen so far, then the suffix scan that picks the next digit.
template <typename T, int SHIFT>
__device__ void radix_level(const T* __restrict__ row, int32_t n, const SampleParams& p, float nk,
                            unsigned long long* s_hist, unsigned long long* s_tot,
                            unsigned long long* s_wave, Select* s_sel, unsigned long long& target) {
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < kBins * kCopies; i += kThreads) s_hist[i] = 0ull;
    __syncthreads();
    const uint32_t prefix = s_sel->prefix;
    Histogram<SHIFT> h{p.k2, nk, prefix, s_hist, (uint32_t)(lane & (kCopies - 1))};
    sweep<T>(row, n, h);
    __syncthreads();
    if (tid < kBins) {  // fold the copies of my bin
        unsigned long long t = 0;
#pragma unroll
        for (int c = 0; c < kCopies; ++c) t += s_hist[tid * kCopies + ((c + tid) & (kCopies - 1))];
        s_tot[tid] = t;
    }
    __syncthreads();
    // thread t owns bin (kBins - 1 - t): descending key order
    const int bin = kBins - 1 - tid;
    scan_select(tid < kBins ? s_tot[bin] : 0ull, (prefix << kRadixBits) | (uint32_t)bin, s_wave, s_sel, target);
}

// The entries whose upper 16 key bits equal `prefix`, copied to a list in LDS (in no particular
// order: what is done with them does not depend on it).  *count ends as the number of such
// entries, also when they do not all fit.
struct GatherPrefix {
    uint32_t prefix;
    float* list;
    int32_t* count;
    int32_t capacity;
    template <int N> __device__ __forceinline__ void run(int32_t, const float (&x)[N], bool) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const bool match = (order_key(x[j]) >> 16) == prefix;
            const unsigned long long mask = __ballot(match);
            if (mask == 0) continue;
            int32_t base = 0;
            if ((threadIdx.x & 63) == 0) base = atomicAdd(count, (int32_t)__popcll(mask));
            base = __builtin_amdgcn_readfirstlane(base);
            const int32_t pos = base + (int32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (match && pos < capacity) list[pos] = x[j];
        }
    }
};

// The upper 16 key bits in one sweep, for rows whose cut lies within kWindowBytes values of the
// key's top byte below the row max (eight binades for four bytes): a histogram over the 16-bit
// key prefixes of that window, one range per thread, and the row's total mass summed per lane
// beside it.  Entries below the window go to a histogram over their key's top byte, so that a
// row whose cut lies there has its first byte-wide level done by the same sweep.
constexpr int kWindowBytes = 4;
constexpr int kWindowBins = kWindowBytes * 256;
constexpr int kWindowCopies = 4;
constexpr int kWindowSlots = kWindowBins * kWindowCopies;
constexpr int kHistSlots = kWindowSlots + kBins * kCopies;  // the window, then the top-byte bins
static_assert(kWindowBins == kThreads, "one window range per thread");
static_assert(kWindowSlots >= kBins * kCopies, "the byte-wide levels reuse the window's slots");

struct WindowHistogram {
    float k2, nk;
    uint32_t top16;            // highest 16-bit prefix of the window
    unsigned long long* hist;  // [kWindowBins][kWindowCopies], then [kBins][kCopies]
    uint32_t lane;
    template <int N> __device__ __forceinline__ void run(int32_t, const float (&x)[N], bool) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t key = order_key(x[j]);
            const uint32_t idx = top16 - (key >> 16);  // no key of the row lies above top16
            const unsigned long long fx = to_fixed40(__builtin_amdgcn_exp2f(fmaf(x[j], k2, nk)));
            const uint32_t fine = idx * kWindowCopies + (lane & (kWindowCopies - 1));
            const uint32_t coarse = kWindowSlots + (key >> 24) * kCopies + (lane & (kCopies - 1));
            atomicAdd(&hist[idx < (uint32_t)kWindowBins ? fine : coarse], fx);
        }
    }
};

// Leaves the upper 16 key bits of the cut in s_sel.  Returns false (the same for every thread)
// when the row has no mass at all.
template <typename T>
__device__ bool window_level(const T* __restrict__ row, const SampleParams& p, float xmax, float nk,
                             unsigned long long* s_hist, unsigned long long* s_tot,
                             unsigned long long* s_wave, Select* s_sel, unsigned long long& target) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < kHistSlots; i += kThreads) s_hist[i] = 0ull;
    __syncthreads();
    const uint32_t top16 = (order_key(xmax) >> 16) | 0xFFu;
    WindowHistogram h{p.k2, nk, top16, s_hist, (uint32_t)lane};
    sweep<T>(row, p.V, h);  // -inf entries and inactive lanes add 0 to some bin
    __syncthreads();
    unsigned long long mine = 0, below = 0;  // my window range; the top-byte bin of my number
#pragma unroll
    for (int c = 0; c < kWindowCopies; ++c) mine += s_hist[tid * kWindowCopies + ((c + tid) & (kWindowCopies - 1))];
    if (tid < kBins) {
#pragma unroll
        for (int c = 0; c < kCopies; ++c) below += s_hist[kWindowSlots + tid * kCopies + ((c + tid) & (kCopies - 1))];
    }
    const unsigned long long total = block_sum_u64(mine + below, s_wave);
    if (total == 0) return false;
    target = top_p_target(p.top_p, total);
    scan_select(mine, top16 - (uint32_t)tid, s_wave, s_sel, target);
    if (s_sel->found) return true;
    // The cut lies below the window.  Top-byte totals: the window's bytes from its ranges (256
    // threads, four waves, each), the others from the top-byte bins; then that byte's level.
    unsigned long long wave_mass = mine;
#pragma unroll
    for (int mask = 1; mask < 64; mask <<= 1) wave_mass += shfl_xor_u64(wave_mass, mask);
    if (lane == 0) s_wave[wave] = wave_mass;
    __syncthreads();
    if (tid < kBins) {
        unsigned long long t = below;
        const uint32_t below_top = (top16 >> 8) - (uint32_t)tid;  // 0 for the window's highest byte
        if (below_top < (uint32_t)kWindowBytes)
            for (int w = 0; w < 4; ++w) t += s_wave[below_top * 4 + w];
        s_tot[tid] = t;
    }
    __syncthreads();
    const int bin = kBins - 1 - tid;
    scan_select(tid < kBins ? s_tot[bin] : 0ull, (uint32_t)bin, s_wave, s_sel, target);
    radix_level<T, 16>(row, p.V, p, nk, s_hist, s_tot, s_wave, s_sel, target);
    return true;
}

// ---- bf16 rows: the cut from a count of every value -----------------------------------------
// A bf16 logit is one of 65536 bit patterns, and all entries of one value have one weight, so
// the cut needs no masses while the row streams by: ONE sweep counts the entries of every value
// (two 16-bit counters per LDS word, 128 KiB), and needs neither the row max nor an exponential
// per entry.  The max is then the highest value with a count, a value's mass is
// count * fixed40(exp(z - max)) (the very integers the histogram route adds up entry by entry, so
// both routes find the same cut), and the values are walked in descending order until the
// running mass reaches ceil(top_p * total): by chunks of 128 values, then inside the chunk that
// crosses.  Chunks without entries (most of the 512) cost a load and a vote.
// A 16-bit counter that overflows (65536 equal entries) is noticed, because the counts no longer
// add up to the number of entries counted, and the row takes the histogram route instead.
// Entries of -inf are not counted (a heavily masked row would overflow their counter).
constexpr int kCountWords = 32768;
constexpr int kCountChunks = kCountWords / 64;  // 512 chunks of 64 words = 128 values
static_assert(kCountChunks <= kThreads && kCountChunks % kWavesPerBlock == 0, "one thread per chunk in the scan");

// The value with 16-bit order key k (the key of order_key() without its lower 16 bits).
__device__ __forceinline__ float key16_value(uint32_t k) {
    const uint32_t b = (k & 0x8000u) ? (k ^ 0x8000u) : (~k & 0xFFFFu);
    return __uint_as_float(b << 16);
}

__device__ __forceinline__ void count_value(uint32_t* cnt, uint32_t f, uint32_t& counted) {
    if (f == 0xFF800000u) return;                                   // -inf: no mass, not counted
    const uint32_t key = f ^ ((uint32_t)((int32_t)f >> 31) | 0x80000000u);   // order key, upper 16 bits used
    atomicAdd(&cnt[key >> 17], 1u + ((key >> 16) & 1u) * 0xFFFFu);   // low or high 16-bit counter
    ++counted;
}

struct CountCut {
    enum { kNoMass = 0, kFound = 1, kOverflow = 2 };
};

// Returns CountCut::kFound with *xmax_out, *xcut_out, *kept_out (the kept set's mass relative to
// the max, 2^-40 fixed point; and *raw_lse_out with RAW) set,
// kNoMass for a row without a finite entry, kOverflow if a counter overflowed (nothing set).
// The same value in every thread.  s_u64: kWavesPerBlock + 2 words; s_u32: 2 * kWavesPerBlock + 2;
// s_f64: kWavesPerBlock; s_chunk: kCountChunks.
template <bool RAW>
__device__ int count_cut_bf16(const uint16_t* __restrict__ row, const SampleParams& p, uint32_t* cnt,
                              unsigned long long* s_u64, uint32_t* s_u32, double* s_f64,
                              unsigned long long* s_chunk, Select* s_sel, float* xmax_out,
                              float* xcut_out, unsigned long long* kept_out, double* raw_lse_out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    {
        uint4* z = (uint4*)cnt;
        for (int i = tid; i < kCountWords / 4; i += kThreads) z[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    __syncthreads();
    // ---- the sweep: one LDS atomic per entry
    uint32_t counted = 0;
    {
        const int32_t nvec = p.V / 8;
        const uint4* __restrict__ row16 = (const uint4*)row;
        const uint4 none = make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u);
        int32_t vi = tid;
        uint4 cur = vi < nvec ? row16[vi] : none;
        for (int32_t base = 0; base < nvec; base += kThreads) {
            const int32_t vn = vi + kThreads;
            const uint4 nxt = vn < nvec ? row16[vn] : none;
            const uint32_t w[4] = {cur.x, cur.y, cur.z, cur.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                count_value(cnt, w[j] << 16, counted);
                count_value(cnt, w[j] & 0xFFFF0000u, counted);
            }
            cur = nxt;
            vi = vn;
        }
        const int32_t i = nvec * 8 + tid;
        if (i < p.V) count_value(cnt, (uint32_t)row[i] << 16, counted);
    }
    __syncthreads();
    // The 65536 values in descending order are 512 chunks of 128 (64 words, the high half of a
    // word before its low half; lane l of the wave that handles chunk c holds word
    // kCountWords - 1 - 64 c - l).  Chunk c is handled by wave c % 16: the few chunks that hold
    // entries lie next to each other, and this way every wave gets some of them.
    constexpr int kIters = kCountChunks / kWavesPerBlock;
    // ---- pass 0: entries counted, which of the wave's chunks hold entries at all (a bit per
    // iteration, the same in every lane) and, from the highest of those, the highest value that
    // has any
    uint32_t busy = 0;
    {
        uint32_t in_bins = 0;
#pragma unroll
        for (int i = 0; i < kIters; ++i) {
            const uint32_t c = cnt[kCountWords - 1 - 64 * (kWavesPerBlock * i + wave) - lane];
            in_bins = __builtin_amdgcn_sad_u16(c, 0u, in_bins);  // + low half + high half
            busy |= __any(c != 0u) ? 1u << i : 0u;
        }
        busy = __builtin_amdgcn_readfirstlane(busy);
        uint32_t top = 0;
        if (busy != 0) {
            const uint32_t word = kCountWords - 1 - 64 * (kWavesPerBlock * __builtin_ctz(busy) + wave) - lane;
            const uint32_t c = cnt[word];
            top = c >> 16 ? 2u * word + 1u : (c ? 2u * word : 0u);
        }
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            in_bins += __shfl_xor(in_bins, mask);
            counted += __shfl_xor(counted, mask);
            const uint32_t o = __shfl_xor(top, mask);
            top = top > o ? top : o;
        }
        if (lane == 0) {
            s_u32[wave] = in_bins;
            s_u32[kWavesPerBlock + wave] = top;
            s_u64[wave] = counted;
        }
        if (tid < kCountChunks) s_chunk[tid] = 0ull;
    }
    __syncthreads();
    uint32_t in_bins = 0, top = 0;
    unsigned long long counted_all = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) {
        in_bins += s_u32[w];
        top = top > s_u32[kWavesPerBlock + w] ? top : s_u32[kWavesPerBlock + w];
        counted_all += s_u64[w];
    }
    __syncthreads();
    if ((unsigned long long)in_bins != counted_all) return CountCut::kOverflow;
    if (counted_all == 0) return CountCut::kNoMass;
    const float xmax = key16_value(top);
    const float nk = ref_offset(xmax, p.k2);
    // mass of one value: count * fixed40(exp(z - max))
    auto mass_of = [&](uint32_t count, uint32_t key) -> unsigned long long {
        return count ? count * to_fixed40(__builtin_amdgcn_exp2f(fmaf(key16_value(key), p.k2, nk))) : 0ull;
    };
    // ---- pass A: the mass of every chunk that holds entries
    {
        double raw = 0.0;
#pragma unroll 1
        for (uint32_t left = busy; left != 0; left &= left - 1) {
            const int32_t chunk = kWavesPerBlock * (__builtin_ctz(left)) + wave;
            const uint32_t word = kCountWords - 1 - 64 * chunk - lane;
            const uint32_t c = cnt[word];
            unsigned long long mine = mass_of(c >> 16, 2u * word + 1u) + mass_of(c & 0xFFFFu, 2u * word);
#pragma unroll
            for (int mask = 1; mask < 64; mask <<= 1) mine += shfl_xor_u64(mine, mask);
            if (RAW) {
                const uint32_t c_hi = c >> 16, c_lo = c & 0xFFFFu;
                raw += (c_hi ? (double)c_hi * (double)__builtin_amdgcn_exp2f((key16_value(2u * word + 1u) - xmax) * kLog2e) : 0.0) +
                       (c_lo ? (double)c_lo * (double)__builtin_amdgcn_exp2f((key16_value(2u * word) - xmax) * kLog2e) : 0.0);
            }
            if (lane == 0) s_chunk[chunk] = mine;
        }
        if (RAW) {
#pragma unroll
            for (int mask = 1; mask < 64; mask <<= 1) raw += shfl_xor_f64(raw, mask);
            if (lane == 0) s_f64[wave] = raw;
        }
    }
    __syncthreads();
    // ---- the chunk at which the running mass reaches the target: the first eight waves scan
    // one chunk per thread
    constexpr int kScanWaves = kCountChunks / 64;
    unsigned long long incl = tid < kCountChunks ? s_chunk[tid] : 0ull;
    const unsigned long long chunk_mass = incl;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long v = shfl_up_u64(incl, d);
        if (lane >= d) incl += v;
    }
    if (lane == 63 && wave < kScanWaves) s_u64[wave] = incl;
    __syncthreads();
    unsigned long long total = 0, base = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        if (w == wave) base = total;
        total += s_u64[w];
    }
    const unsigned long long target = top_p_target(p.top_p, total);
    if (wave < kScanWaves && base + incl - chunk_mass < target && base + incl >= target) {
        s_sel->prefix = (uint32_t)tid;                // the chunk
        s_sel->above = base + incl - chunk_mass;      // mass of all chunks above it
    }
    __syncthreads();
    // ---- pass B: the wave of that chunk finds the value inside it
    const int32_t cross = (int32_t)s_sel->prefix;
    if (wave == (cross & (kWavesPerBlock - 1))) {
        const uint32_t word = kCountWords - 1 - 64 * cross - lane;
        const uint32_t c = cnt[word];
        const unsigned long long hi = mass_of(c >> 16, 2u * word + 1u), lo = mass_of(c & 0xFFFFu, 2u * word);
        const unsigned long long m = hi + lo;
        unsigned long long run = m;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned long long v = shfl_up_u64(run, d);
            if (lane >= d) run += v;
        }
        run += s_sel->above;                             // mass of this lane's values and all higher ones
        const unsigned long long before = run - m;
        if (before < target && run >= target) {
            const bool in_hi = before + hi >= target;    // hi > 0 then, since before < target
            const uint32_t kcut = in_hi ? 2u * word + 1u : 2u * word;
            unsigned long long kept = in_hi ? before + hi : run;
            // -0 and +0 are one value with two bit patterns, -0 (key 0x7FFF) right below +0 (key
            // 0x8000): a cut at +0 keeps the entries of -0 too.  (A cut at -0 keeps +0 anyway.)
            if (kcut == 0x8000u) kept += mass_of(cnt[0x3FFF] >> 16, 0x7FFFu);
            s_u32[0] = kcut;
            s_u64[kWavesPerBlock] = kept;
        }
    }
    __syncthreads();
    if (tid == 0) {
        *xmax_out = xmax;
        *xcut_out = key16_value(s_u32[0]);
        *kept_out = s_u64[kWavesPerBlock];
        if (RAW) {
            double sr = 0.0;
            for (int w = 0; w < kWavesPerBlock; ++w) sr += s_f64[w];
            *raw_lse_out = (double)xmax + log(sr);
        }
    }
    __syncthreads();
    return CountCut::kFound;
}

// RAW: also accumulate sum exp(x - max) at temperature 1 for raw_logprob_out (needed only when
// the sampled distribution differs from the raw one).
template <typename T, bool TOPP, bool RAW>
__global__ __launch_bounds__(kThreads) void sample_rows(const T* __restrict__ logits,
                                                         const int32_t* __restrict__ row_ids,
                                                         int32_t* __restrict__ tokens_out,
                                                         float* __restrict__ logprob_out,
                                                         float* __restrict__ raw_logprob_out, SampleParams p) {
    // bf16 rows with top-p count every value first (count_cut_bf16): 128 KiB of counters, which
    // the histogram route and the race's queues then reuse.
    constexpr bool kCounts = TOPP && std::is_same<T, uint16_t>::value;
    constexpr int kBigWords = kCounts ? kCountWords / 2 : (TOPP ? kHistSlots : 1);
    __shared__ __align__(16) unsigned long long s_hist[kBigWords];
    __shared__ unsigned long long s_tot[TOPP ? kBins : 1];
    __shared__ unsigned long long s_wave[kWavesPerBlock + 2];
    __shared__ uint32_t s_u32[2 * kWavesPerBlock + 2];
    __shared__ unsigned long long s_chunk[kCounts ? kCountChunks : 1];
    __shared__ Select s_sel;
    __shared__ float s_m[kWavesPerBlock];
    __shared__ double s_s[kWavesPerBlock];
    __shared__ double s_best[kWavesPerBlock];
    __shared__ int32_t s_besti[kWavesPerBlock];
    __shared__ float s_xcut;
    __shared__ unsigned long long s_kept;  // top-p: mass of the kept set relative to the row max, 2^-40 fixed point
    __shared__ double s_lse;
    __shared__ double s_sraw[kWavesPerBlock];
    __shared__ double s_raw_lse;
    __shared__ uint32_t s_thr_key;
    __shared__ int32_t s_count;

    const int32_t r = blockIdx.x;
    const T* __restrict__ row = logits + (int64_t)r * p.row_stride;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row_id = row_ids ? (uint32_t)row_ids[r] : (uint32_t)r;

    if (threadIdx.x == 0) s_thr_key = order_key(-INFINITY);
    __syncthreads();

    // Block max of the raw logits from the threads' maxima and, for top_p == 1, the log-sum-exp in
    // log2 units of the logits times k2: a lane's sum is relative to 2^(-nk) of its own reference,
    // the block's to that of the row max, and the sampled token's log-prob is taken with the same
    // k2, so the rounding of k2 and of nk cancels (a row with all its mass on one entry gives 0).
    // Leaves the max in s_m[0], the log-sum-exp in s_lse and the raw one in s_raw_lse.
    auto reduce_max_and_sums = [&](float mine, float s_thread, float nk_thread, float s_raw_thread) {
        float m = mine;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) m = fmaxf(m, __shfl_xor(m, mask));
        double s = TOPP ? 0.0 : (double)s_thread * (double)__builtin_amdgcn_exp2f(ref_offset(m, p.k2) - nk_thread);
        double sr = (double)s_raw_thread * (double)__builtin_amdgcn_exp2f((mine - m) * kLog2e);
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            s += shfl_xor_f64(s, mask);
            sr += shfl_xor_f64(sr, mask);
        }
        if (lane == 0) { s_m[wave] = m; s_s[wave] = s; s_sraw[wave] = sr; }
        __syncthreads();
        if (tid == 0) {
            float M = s_m[0];
            for (int w = 1; w < kWavesPerBlock; ++w) M = fmaxf(M, s_m[w]);
            double S = 0.0, SR = 0.0;
            for (int w = 0; w < kWavesPerBlock; ++w) {
                S += s_s[w] * (double)__builtin_amdgcn_exp2f(ref_offset(M, p.k2) - ref_offset(s_m[w], p.k2));
                SR += s_sraw[w] * (double)__builtin_amdgcn_exp2f((s_m[w] - M) * kLog2e);
            }
            s_m[0] = M;
            s_lse = (log2(S) - (double)ref_offset(M, p.k2)) / kLog2ed;
            s_raw_lse = (double)M + log(SR);
            s_sel.prefix = 0;
            s_sel.above = 0;
        }
        __syncthreads();
    };

    Race<true, RAW, false> race{p, row_id, -INFINITY, -FLT_MAX};
    Race<false, false, true> race_kept{p, row_id, -INFINITY, 0.f};
    if constexpr (!TOPP) {
        race.block_thr_key = &s_thr_key;
        race.set_ref(-FLT_MAX);
        sweep<T>(row, p.V, race);  // one sweep: online log-sum-exp and the race together
        reduce_max_and_sums(race.xref, race.s, race.nk, race.s_raw);
    } else {
        // The cut: s_m[0] = row max, s_xcut, s_kept (the kept set's mass; its logarithm is taken at
        // the end, beside the load of the winner's logit) and s_raw_lse.
        bool has_mass = false, have_cut = false;
        if constexpr (kCounts) {
            const int st = count_cut_bf16<RAW>(row, p, (uint32_t*)s_hist, s_wave, s_u32, s_s, s_chunk, &s_sel, &s_m[0],
                                               &s_xcut, &s_kept, &s_raw_lse);
            have_cut = st != CountCut::kOverflow;
            has_mass = st == CountCut::kFound;
        }
        if (!have_cut) {
            // The histogram route: a sweep for the row max, the upper 16 key bits from the window
            // sweep (and a sweep for the second byte when the cut lies below the window), then the
            // lower 16 of an fp32 key.  A row without mass (no finite entry) has no cut and no race:
            // the result below is then "no token".
            MaxOnly<RAW> mo;
            sweep<T>(row, p.V, mo);
            reduce_max_and_sums(mo.xm, 0.f, 0.f, mo.s_raw);
            const float xM = s_m[0];
            const float nkM = ref_offset(xM, p.k2);
            constexpr int kKeyBits = Elem<T>::kKeyBits;
            unsigned long long target = 0;
            has_mass = window_level<T>(row, p, xM, nkM, s_hist, s_tot, s_wave, &s_sel, target);
            if (has_mass) {
                if constexpr (kKeyBits == 32) {
                    // The lower 16 key bits concern only the entries that share the upper 16 with the
                    // cut, usually a few hundred: they are gathered into LDS in one sweep and the two
                    // byte-wide levels run over that list.  Rows with more such entries than the list
                    // holds (many equal logits) take the levels over the whole row.
                    constexpr int32_t kListCap = (kHistSlots - kBins * kCopies) * 2;  // floats behind the level's bins
                    float* list = (float*)(s_hist + kBins * kCopies);
                    if (tid == 0) s_count = 0;
                    __syncthreads();
                    GatherPrefix g{s_sel.prefix, list, &s_count, kListCap};
                    sweep<T>(row, p.V, g);
                    __syncthreads();
                    const int32_t n_list = s_count;
                    const T* src = n_list <= kListCap ? (const T*)list : row;
                    const int32_t n_src = n_list <= kListCap ? n_list : p.V;
                    radix_level<T, 8>(src, n_src, p, nkM, s_hist, s_tot, s_wave, &s_sel, target);
                    radix_level<T, 0>(src, n_src, p, nkM, s_hist, s_tot, s_wave, &s_sel, target);
                }
                if (tid == 0) {
                    // s_sel.prefix is now the key of the cut value (its upper 16 bits for bf16, whose
                    // lower key bits are all ones for negative values and zero otherwise).  The kept
                    // mass is everything above the cut plus the cut value's own class.
                    const uint32_t key = (s_sel.prefix << (32 - kKeyBits)) |
                                         (kKeyBits == 16 ? ((s_sel.prefix >> 15) ? 0u : 0xFFFFu) : 0u);
                    s_xcut = key_to_float(key);
                    s_kept = s_sel.kept;
                }
                __syncthreads();
            }
        }
        if (has_mass) {
            race_kept.block_thr_key = &s_thr_key;  // still -inf: no race has run in this launch
            race_kept.x_cut = s_xcut;
            race_kept.set_ref(s_m[0]);
            race_kept.refresh_c();
            static_assert(kWavesPerBlock * kQueueBytesPerWave <= kBigWords * 8, "the queues reuse the histogram");
            CompactRace<Race<false, false, true>> gathered{
                race_kept, (float*)s_hist + wave * (kQueueCap * 4),
                (uint32_t*)s_hist + kWavesPerBlock * (kQueueCap * 4) + wave * kQueueCap};
            sweep<T>(row, p.V, gathered);
            gathered.finish();
        }
    }

    // Block arg-max of the exact perturbed values (lowest index on ties).
    {
        double b = TOPP ? race_kept.best : race.best;
        int32_t bi = TOPP ? race_kept.best_i : race.best_i;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            const double ob = shfl_xor_f64(b, mask);
            const int32_t oi = __shfl_xor(bi, mask);
            if (ob > b || (ob == b && oi < bi)) { b = ob; bi = oi; }
        }
        if (lane == 0) { s_best[wave] = b; s_besti[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kWavesPerBlock; ++w)
                if (s_best[w] > b || (s_best[w] == b && s_besti[w] < bi)) { b = s_best[w]; bi = s_besti[w]; }
            if (p.policy_version_out) p.policy_version_out[r] = p.policy_version;
            if ((uint32_t)bi >= (uint32_t)p.V) {  // no finite entry in the row
                tokens_out[r] = -1;
                logprob_out[r] = NAN;
                if (raw_logprob_out) raw_logprob_out[r] = NAN;
            } else {
                tokens_out[r] = bi;
                const T x_bits = row[bi];
                const double lse = TOPP ? (log2((double)s_kept * 0x1p-40) - (double)ref_offset(s_m[0], p.k2)) / kLog2ed : s_lse;
                const double x = (double)Elem<T>::widen(x_bits);
                const float lp = (float)(x * (double)p.k2 / kLog2ed - lse);
                logprob_out[r] = lp;
                // without an extra sum the sampled distribution is the raw one (T = 1, top_p = 1)
                if (raw_logprob_out) raw_logprob_out[r] = RAW ? (float)(x - s_raw_lse) : lp;
            }
        }
    }
}

int validate(const roll_sample_desc* d) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->batch <= 0 || d->vocab <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "batch and vocab must be > 0");
    if (d->row_stride < d->vocab) return roll::fail(ROLL_ERR_INVALID_ARG, "row_stride < vocab");
    if (d->logits_dtype != ROLL_BF16 && d->logits_dtype != ROLL_F32) return roll::fail(ROLL_ERR_INVALID_ARG, "logits_dtype must be ROLL_BF16 or ROLL_F32");
    const int64_t elem = d->logits_dtype == ROLL_BF16 ? 2 : 4;
    if ((d->row_stride * elem) % 16 != 0) return roll::fail(ROLL_ERR_INVALID_ARG, "rows must start 16-byte aligned (row_stride * element size %% 16 == 0)");
    return ROLL_OK;
}

}  // namespace

extern "C" size_t roll_sample_logprob_workspace_bytes(const roll_sample_desc* d) {
    if (validate(d) != ROLL_OK) return 0;
    return 256;  // reserved; the current kernels keep all intermediate state on chip
}

extern "C" int roll_sample_logprob(const void* logits, float temperature, float top_p,
                                   uint64_t philox_seed, uint64_t step, int32_t* tokens_out,
                                   float* logprob_out, const roll_sample_desc* d, void* workspace,
                                   size_t workspace_bytes, void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    if (!logits || !tokens_out || !logprob_out) return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(logits, 16)) return roll::fail(ROLL_ERR_INVALID_ARG, "logits must be 16-byte aligned");
    if (!(temperature > 0.f) || std::isinf(temperature)) return roll::fail(ROLL_ERR_INVALID_ARG, "temperature must be finite and > 0");
    if (!(top_p > 0.f) || top_p > 1.f) return roll::fail(ROLL_ERR_INVALID_ARG, "top_p must be in (0, 1]");
    (void)workspace;
    (void)workspace_bytes;
    hipStream_t stream = (hipStream_t)stream_v;
    SampleParams p{};
    p.V = d->vocab;
    p.row_stride = d->row_stride;
    p.k2 = (float)(1.44269504088896340736 / (double)temperature);
    p.temperature = (double)temperature;
    p.top_p = top_p;
    p.seed_lo = (uint32_t)philox_seed;
    p.seed_hi = (uint32_t)(philox_seed >> 32);
    p.step_lo = (uint32_t)step;
    p.step_hi = (uint32_t)(step >> 32);
    p.policy_version = d->policy_version;
    p.policy_version_out = d->policy_version_out;
    const bool topp = top_p < 1.0f;
    float* raw = d->raw_logprob_out;
    const bool raw_sum = raw != nullptr && (topp || temperature != 1.0f);
    const dim3 grid(d->batch), block(kThreads);
    const int variant = (d->logits_dtype == ROLL_BF16 ? 0 : 4) + (topp ? 2 : 0) + (raw_sum ? 1 : 0);
#define ROLL_LAUNCH_SAMPLE(T, TOPP, RAW)                                                            \
    sample_rows<T, TOPP, RAW><<<grid, block, 0, stream>>>((const T*)logits, d->row_ids, tokens_out, \
                                                          logprob_out, raw, p)
    switch (variant) {
        case 0: ROLL_LAUNCH_SAMPLE(uint16_t, false, false); break;
        case 1: ROLL_LAUNCH_SAMPLE(uint16_t, false, true); break;
        case 2: ROLL_LAUNCH_SAMPLE(uint16_t, true, false); break;
        case 3: ROLL_LAUNCH_SAMPLE(uint16_t, true, true); break;
        case 4: ROLL_LAUNCH_SAMPLE(float, false, false); break;
        case 5: ROLL_LAUNCH_SAMPLE(float, false, true); break;
        case 6: ROLL_LAUNCH_SAMPLE(float, true, false); break;
        default: ROLL_LAUNCH_SAMPLE(float, true, true); break;
    }
#undef ROLL_LAUNCH_SAMPLE
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}
