// Consumer of the recorded behaviour-policy log-probs: the off-policy objectives and the
// truncated importance weight, over ragged responses.
//
// ROLL Flash (arXiv 2510.11345) Section 3.2 lists five per-token objectives (PPO, Decoupled PPO,
// Truncated IS, CISPO, TOPR) over pi_theta, pi_old (the rollout engine's probability, which the
// decode step records) and pi_prox; Appendix A.1 caps the importance weight pi_train / pi_rollout
// at C.  The kernel evaluates the chosen objective and its derivative with respect to
// log pi_theta for every token (what a trainer multiplies into grad log pi), the truncated weight
// min(r, c), the per-response mean (1/|o|) sum_t and the mean over responses.
//
// 16-20 bytes in and up to 12 bytes out per token, and about 80 vector instructions (the fp64
// exponential half of them).  The tokens of the whole batch, laid end to end, are cut into shares
// of 1024 tokens (larger ones only for batches above 2^26 tokens) whatever the lengths of the
// responses, and the waves of a fixed grid (16 per compute unit) take the shares round-robin: the
// longest response of a long-tailed batch is then spread over many waves instead of being one
// workgroup's work, and at any moment the grid reads and writes one contiguous window of every
// array (neighbouring waves hold neighbouring shares), which DRAM serves far better than
// thousands of distant streams.  A wave streams a share in rounds of 256 tokens, the loads of the
// next round in flight while the current one is computed, and attributes every token's value to
// the response it belongs to as it goes.  A response that lies inside the share gets its mean
// from that wave alone, a response that crosses shares leaves one partial sum per share in the
// workspace (at most two per share: the response that began before the share and the one that
// continues after it), and the second kernel adds them up in share order and forms the batch
// mean.  All sums are fp64 in a fixed order, so results are reproducible.  The ratios and the
// branch decisions of min / clip are taken in fp64 from the fp32 inputs, the precision the
// definition is stated in.
#include <cmath>

#include "common.h"

namespace {

constexpr int kUnroll = 4;        // tokens per thread and round

struct LossParams {
    int32_t kind;
    double eps_lo, eps_hi, c;
};

__device__ __forceinline__ double clipd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

__device__ __forceinline__ void loss_token(const LossParams& p, double lt, double lo, double lp, double R,
                                           double& v, double& g, double& w) {
    const double r = exp(lt - lo);
    w = r < p.c ? r : p.c;
    if (p.kind == ROLL_LOSS_PPO || p.kind == ROLL_LOSS_DECOUPLED_PPO) {
        // second branch: R * (pi_prox / pi_old) * clip(pi_theta / pi_prox); pi_prox = pi_old for PPO
        const double rp = p.kind == ROLL_LOSS_PPO ? r : exp(lt - lp);
        const double wp = p.kind == ROLL_LOSS_PPO ? 1.0 : exp(lp - lo);
        const double a = R * r, b = R * wp * clipd(rp, 1.0 - p.eps_lo, 1.0 + p.eps_hi);
        const bool inside = rp > 1.0 - p.eps_lo && rp < 1.0 + p.eps_hi;
        if (a <= b) { v = a; g = R * r; } else { v = b; g = inside ? R * wp * rp : 0.0; }
        return;
    }
    double coef;
    if (p.kind == ROLL_LOSS_TIS) coef = clipd(r, 0.0, p.c);
    else if (p.kind == ROLL_LOSS_CISPO) coef = clipd(r, 1.0 - p.eps_lo, 1.0 + p.eps_hi);
    else coef = R > 0.0 ? 1.0 : clipd(r, 0.0, p.c);  // TOPR: truncate only the low-return set
    v = coef * R * lt;
    g = coef * R;
}

constexpr int kWavesPerGroup = 4;                 // 256-thread workgroups
constexpr int kWavesPerCu = 16;
constexpr int kRound = 64 * kUnroll;              // tokens of a wave's round
constexpr int kShareTokens = 4 * kRound;          // tokens per share, unless the batch is huge
constexpr int kMaxShares = 65536;                 // the workspace holds two sums per share
constexpr size_t kLossWorkspaceBytes = sizeof(double) * 2 * kMaxShares + 256;  // two sums per share, an arrival counter
constexpr int kLdsOffsets = 8191;                 // response offsets (one more entry) staged in 64 KiB of LDS when they fit

struct Shares {
    int64_t T;      // tokens in the batch
    int64_t size;   // tokens per share, a multiple of the round
    int64_t S;      // shares
    __device__ explicit Shares(int64_t tokens) : T(tokens) {
        const int64_t least = (tokens + kMaxShares - 1) / kMaxShares;   // share size that keeps S <= kMaxShares
        size = least <= kShareTokens ? kShareTokens : (least + kRound - 1) / kRound * kRound;
        S = (tokens + size - 1) / size;
    }
    __device__ int64_t start(int64_t sh) const { const int64_t x = sh * size; return x < T ? x : T; }
    __device__ int64_t owner(int64_t t) const { return t / size; }   // the share that holds token t
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int mask = 1; mask < 64; mask <<= 1) {
        const uint64_t b = __builtin_bit_cast(uint64_t, v);
        const uint32_t lo = __shfl_xor((uint32_t)b, mask), hi = __shfl_xor((uint32_t)(b >> 32), mask);
        v += __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
    }
    return v;
}

struct TokenRound {  // the inputs of kUnroll tokens of a lane
    float t[kUnroll], o[kUnroll], p[kUnroll], r[kUnroll];
};

// Inside a share tokens are addressed by 32-bit offsets from the share's first token (a share is
// the batch's 1/W: below 2^30 tokens for any batch that fits a GPU), so that the four input
// arrays and the three output arrays share one offset computation per token and every compare of
// the walk is one instruction.
constexpr uint32_t kLocalMax = 0x3FFFFFFFu;
__device__ __forceinline__ uint32_t to_local(int64_t x) { return x < 0 ? 0u : (x > (int64_t)kLocalMax ? kLocalMax : (uint32_t)x); }

template <typename T>
__device__ __forceinline__ T& at_bytes(T* base, uint32_t byte_offset) { return *(T*)((char*)base + byte_offset); }

// Lane's tokens of the round that begins at local offset `begin`: begin + lane + 64 u.  Offsets
// past `last` (the batch's last token) are clamped to it, so every load is unconditional (a load
// inside a branch makes the compiler wait for all earlier loads where the branch joins, one round
// trip after the other); what the clamped lanes compute is discarded by the caller.
template <bool PROX>
__device__ __forceinline__ void load_round(TokenRound& d, const float* __restrict__ lt, const float* __restrict__ lo,
                                           const float* __restrict__ lp, const float* __restrict__ R, uint32_t begin,
                                           uint32_t last, int32_t lane) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        uint32_t j = begin + lane + 64 * u;
        j = (j < last ? j : last) * 4u;
        d.t[u] = at_bytes(lt, j);
        d.o[u] = at_bytes(lo, j);
        d.p[u] = PROX ? at_bytes(lp, j) : 0.f;
        d.r[u] = at_bytes(R, j);
    }
}

// head[sh]: sum over the tokens, inside share sh, of the response that began before the share
// (0 if none); tail[sh]: of the response that begins inside the share and continues after it.
// STAGED: the response offsets are read from LDS.  The address space has to be known at compile
// time: through a pointer that may be either, every read becomes a flat load, which counts as a
// vector-memory load too and so waits for the token loads in flight ahead of it.
template <bool PROX, bool STAGED>
__global__ __launch_bounds__(kWavesPerGroup * 64) void policy_loss_tokens(
    const float* __restrict__ lt, const float* __restrict__ lo, const float* __restrict__ lp,
    const float* __restrict__ R, const int64_t* __restrict__ offsets, int32_t n_seq, float* __restrict__ value,
    float* __restrict__ grad, float* __restrict__ is_weight, float* __restrict__ seq_mean,
    double* __restrict__ head, double* __restrict__ tail, uint32_t* __restrict__ arrivals, int32_t W, LossParams p) {
    extern __shared__ int64_t s_off[];  // offsets[0 .. n_seq] when STAGED
    if (blockIdx.x == 0 && threadIdx.x == 0) *arrivals = 0u;  // for the second kernel
    auto off = [&](int32_t i) -> int64_t { return STAGED ? s_off[i] : offsets[i]; };
    const int32_t lane = threadIdx.x & 63;
    const int32_t w = blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
    const Shares shares(offsets[n_seq]);
    if (STAGED) {
        for (int32_t i = threadIdx.x; i <= n_seq; i += blockDim.x) s_off[i] = offsets[i];
        __syncthreads();
    }
    for (int64_t sh = w; sh < shares.S; sh += W) {
        const int64_t a = shares.start(sh), b = shares.start(sh + 1);
        const uint32_t n = to_local(b - a);               // tokens of the share (> 0)
        const uint32_t last = to_local(shares.T - 1 - a);  // the batch's last token, seen from the share
        // the share's arrays
        const float* const lt_a = lt + a;
        const float* const lo_a = lo + a;
        const float* const lp_a = PROX ? lp + a : nullptr;
        const float* const R_a = R + a;
        float* const value_a = value ? value + a : nullptr;
        float* const grad_a = grad ? grad + a : nullptr;
        float* const weight_a = is_weight ? is_weight + a : nullptr;
        // the first round's loads go out before anything else: they depend on the share alone
        TokenRound cur;
        load_round<PROX>(cur, lt_a, lo_a, lp_a, R_a, 0u, last, lane);
        double head_sum = 0.0, tail_sum = 0.0;
        // the response that holds token a: the last s with off[s] <= a (responses without tokens
        // at that offset come before it and are skipped)
        int32_t s_lo = 0, s_hi = n_seq;  // off[s_lo] <= a < off[s_hi]
        while (s_hi - s_lo > 1) {
            const int32_t mid = (s_lo + s_hi) >> 1;
            if (off(mid) <= a) s_lo = mid; else s_hi = mid;
        }
        int32_t s = s_lo;
        int64_t s_begin = off(s), s_end = off(s + 1);
        uint32_t s_end_l = to_local(s_end - a);  // where response s ends, seen from the share (clamped far beyond it)
        double acc = 0.0;  // this lane's sum over the tokens of response s seen so far
        for (uint32_t begin = 0; begin < n; begin += kRound) {
            TokenRound nxt;
            load_round<PROX>(nxt, lt_a, lo_a, lp_a, R_a, begin + kRound, last, lane);
            const uint32_t round_end = begin + kRound < n ? begin + kRound : n;
            double v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint32_t j = begin + lane + 64 * u;
                double g, wgt;
                loss_token(p, (double)cur.t[u], (double)cur.o[u], (double)(PROX ? cur.p[u] : cur.o[u]), (double)cur.r[u],
                           v[u], g, wgt);
                if (j < n) {
                    if (value_a) at_bytes(value_a, j * 4u) = (float)v[u];
                    if (grad_a) at_bytes(grad_a, j * 4u) = (float)g;
                    if (weight_a) at_bytes(weight_a, j * 4u) = (float)wgt;
                } else {
                    v[u] = 0.0;
                }
            }
            // Every token's value goes to the response that holds it.  The usual round lies inside
            // one response; otherwise the responses that end inside the round are finished one
            // after the other and the last one keeps accumulating.
            if (s_end_l > round_end && round_end < n) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) acc += v[u];
            } else {
                uint32_t from = begin;
                while (true) {
                    const uint32_t seg_end = s_end_l < round_end ? s_end_l : round_end;
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        const uint32_t j = begin + lane + 64 * u;
                        acc += j >= from && j < seg_end ? v[u] : 0.0;
                    }
                    const bool response_ends = s_end_l <= round_end;
                    if (response_ends || round_end == n) {  // the share holds nothing more of response s
                        const double total = wave_sum(acc);
                        acc = 0.0;
                        const bool begins_here = s_begin >= a;
                        if (begins_here && response_ends) {
                            if (lane == 0) seq_mean[s] = (float)(total / (double)(s_end - s_begin));
                        } else if (!begins_here) {
                            head_sum = total;
                        } else {
                            tail_sum = total;
                        }
                    }
                    if (!response_ends || seg_end >= n) break;
                    // the response ended before the share does: on to the next one that has tokens
                    from = seg_end;
                    do { ++s; } while (s < n_seq - 1 && off(s + 1) == off(s));
                    s_begin = off(s);
                    s_end = off(s + 1);
                    s_end_l = to_local(s_end - a);
                    if (seg_end >= round_end) break;
                }
            }
            cur = nxt;
        }
        if (lane == 0) {
            head[sh] = head_sum;
            tail[sh] = tail_sum;
        }
    }
}

// Means of the responses that are empty or cross shares (a thread per response, the grid's
// workgroups side by side), then, by the workgroup that finishes last, the mean of the
// per-response means over the non-empty responses: always summed in the same order, whichever
// workgroup that is.  *arrivals is zero on entry (policy_loss_tokens clears it) and zero again on exit.
constexpr int kMeansThreads = 256;
__global__ __launch_bounds__(kMeansThreads) void policy_loss_means(const int64_t* __restrict__ offsets, int32_t n_seq,
                                                                    float* seq_mean, const double* __restrict__ head,
                                                                    const double* __restrict__ tail,
                                                                    uint32_t* arrivals, float* __restrict__ out) {
    __shared__ double s_sum[kMeansThreads];
    __shared__ int32_t s_cnt[kMeansThreads];
    __shared__ uint32_t s_last;
    const Shares sh(offsets[n_seq]);
    for (int32_t s = blockIdx.x * kMeansThreads + threadIdx.x; s < n_seq; s += gridDim.x * kMeansThreads) {
        const int64_t begin = offsets[s], end = offsets[s + 1];
        if (end <= begin) {
            seq_mean[s] = 0.f;
            continue;
        }
        const int64_t w_first = sh.owner(begin), w_last = sh.owner(end - 1);
        if (w_first == w_last) continue;  // written by the wave of that share
        // in share order, eight loads in flight at a time
        double total = tail[w_first];
        int64_t w = w_first + 1;
        for (; w + 8 <= w_last + 1; w += 8) {
            double h[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) h[k] = head[w + k];
#pragma unroll
            for (int k = 0; k < 8; ++k) total += h[k];
        }
        for (; w <= w_last; ++w) total += head[w];
        seq_mean[s] = (float)(total / (double)(end - begin));
    }
    // the last workgroup to get here sees every other one's means
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t before = __hip_atomic_fetch_add(arrivals, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        s_last = before == gridDim.x - 1;
        if (s_last) __hip_atomic_store(arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    // (plain loads: the fence above has discarded what this workgroup's caches held of seq_mean)
    double acc = 0.0;
    int32_t cnt = 0;
    for (int32_t base = threadIdx.x; base < n_seq; base += 4 * kMeansThreads) {
        float m[4];
        bool live[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t s = base + k * kMeansThreads;
            const int32_t sc = s < n_seq ? s : n_seq - 1;
            live[k] = s < n_seq && offsets[sc + 1] > offsets[sc];
            m[k] = seq_mean[sc];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (live[k]) {
                acc += (double)m[k];
                ++cnt;
            }
    }
    s_sum[threadIdx.x] = acc;
    s_cnt[threadIdx.x] = cnt;
    __syncthreads();
    for (int stride = kMeansThreads / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) {
            s_sum[threadIdx.x] += s_sum[threadIdx.x + stride];
            s_cnt[threadIdx.x] += s_cnt[threadIdx.x + stride];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = s_cnt[0] ? (float)(s_sum[0] / s_cnt[0]) : 0.f;
}

}  // namespace

extern "C" size_t roll_policy_loss_workspace_bytes(const roll_loss_desc* d) {
    if (!d || d->num_seqs <= 0) return 0;
    return kLossWorkspaceBytes;
}

extern "C" int roll_policy_loss(const float* logp_theta, const float* logp_old, const float* logp_prox,
                                const float* signal, const int64_t* seq_offsets, float* value_out,
                                float* grad_out, float* is_weight_out, float* seq_mean_out,
                                float* batch_mean_out, const roll_loss_desc* d, void* workspace,
                                size_t workspace_bytes, void* stream_v) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->kind < ROLL_LOSS_PPO || d->kind > ROLL_LOSS_TOPR) return roll::fail(ROLL_ERR_INVALID_ARG, "unknown objective %d", d->kind);
    if (d->num_seqs <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "num_seqs must be > 0");
    if (!logp_theta || !logp_old || !signal || !seq_offsets || !seq_mean_out || !batch_mean_out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (d->kind == ROLL_LOSS_DECOUPLED_PPO && !logp_prox)
        return roll::fail(ROLL_ERR_INVALID_ARG, "Decoupled PPO needs logp_prox");
    if (!(d->eps_low >= 0.f) || !(d->eps_high >= 0.f) || !(d->c > 0.f))
        return roll::fail(ROLL_ERR_INVALID_ARG, "eps_low, eps_high must be >= 0 and c > 0");
    if (!workspace || !roll::aligned(workspace, 8)) return roll::fail(ROLL_ERR_WORKSPACE, "workspace NULL or not 8-byte aligned");
    if (workspace_bytes < kLossWorkspaceBytes)
        return roll::fail(ROLL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes,
                          kLossWorkspaceBytes);
    LossParams p{d->kind, (double)d->eps_low, (double)d->eps_high, (double)d->c};
    hipStream_t stream = (hipStream_t)stream_v;
    int dev = 0, cus = 0;
    ROLL_HIP_CHECK(hipGetDevice(&dev));
    ROLL_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int32_t W = kWavesPerCu * (cus > 0 ? cus : 256);
    double* head = (double*)workspace;
    double* tail = head + kMaxShares;
    uint32_t* arrivals = (uint32_t*)(tail + kMaxShares);
    const size_t lds = d->num_seqs <= kLdsOffsets ? sizeof(int64_t) * ((size_t)d->num_seqs + 1) : 0;
    const dim3 grid((W + kWavesPerGroup - 1) / kWavesPerGroup), block(kWavesPerGroup * 64);
    const bool prox = d->kind == ROLL_LOSS_DECOUPLED_PPO, staged = d->num_seqs <= kLdsOffsets;
#define ROLL_LAUNCH_LOSS(PROX, STAGED)                                                                       \
    policy_loss_tokens<PROX, STAGED><<<grid, block, lds, stream>>>(                                          \
        logp_theta, logp_old, PROX ? logp_prox : nullptr, signal, seq_offsets, d->num_seqs, value_out, grad_out, \
        is_weight_out, seq_mean_out, head, tail, arrivals, W, p)
    if (prox && staged) ROLL_LAUNCH_LOSS(true, true);
    else if (prox) ROLL_LAUNCH_LOSS(true, false);
    else if (staged) ROLL_LAUNCH_LOSS(false, true);
    else ROLL_LAUNCH_LOSS(false, false);
#undef ROLL_LAUNCH_LOSS
    ROLL_HIP_CHECK(hipGetLastError());
    const int32_t mean_groups = (d->num_seqs + kMeansThreads - 1) / kMeansThreads;
    policy_loss_means<<<mean_groups < 256 ? mean_groups : 256, kMeansThreads, 0, stream>>>(
        seq_offsets, d->num_seqs, seq_mean_out, head, tail, arrivals, batch_mean_out);
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}
