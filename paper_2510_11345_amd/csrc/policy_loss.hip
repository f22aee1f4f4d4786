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
// HBM-bound and tiny: 16-20 bytes in and up to 12 bytes out per token, one workgroup per
// response (a thread strides over its tokens, fixed reduction order, so results are
// reproducible).  The ratios and the branch decisions of min / clip are taken in fp64 from the
// fp32 inputs, the precision the definition is stated in; the arithmetic is nowhere near the
// bandwidth bound.
#include <cmath>

#include "common.h"

namespace {

constexpr int kLossThreads = 1024;
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

__global__ __launch_bounds__(kLossThreads) void policy_loss_rows(
    const float* __restrict__ lt, const float* __restrict__ lo, const float* __restrict__ lp,
    const float* __restrict__ R, const int64_t* __restrict__ offsets, float* __restrict__ value,
    float* __restrict__ grad, float* __restrict__ is_weight, float* __restrict__ seq_mean, LossParams p) {
    __shared__ double s_part[kLossThreads];
    const int32_t s = blockIdx.x;
    const int64_t begin = offsets[s], end = offsets[s + 1];
    double acc = 0.0;
    // kUnroll tokens per thread and round, all loads of a round issued before the arithmetic:
    // the longest response of a long-tailed batch is one workgroup's work, so its time is set
    // by how many bytes that workgroup keeps in flight.
    for (int64_t base = begin + threadIdx.x; base < end; base += (int64_t)kLossThreads * kUnroll) {
        float a_t[kUnroll], a_o[kUnroll], a_p[kUnroll], a_r[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kLossThreads;
            const bool in = i < end;
            a_t[u] = in ? lt[i] : 0.f;
            a_o[u] = in ? lo[i] : 0.f;
            a_p[u] = in && lp ? lp[i] : a_o[u];
            a_r[u] = in ? R[i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kLossThreads;
            if (i >= end) continue;
            double v, g, w;
            loss_token(p, (double)a_t[u], (double)a_o[u], (double)a_p[u], (double)a_r[u], v, g, w);
            if (value) value[i] = (float)v;
            if (grad) grad[i] = (float)g;
            if (is_weight) is_weight[i] = (float)w;
            acc += v;
        }
    }
    s_part[threadIdx.x] = acc;
    __syncthreads();
    for (int stride = kLossThreads / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) s_part[threadIdx.x] += s_part[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) seq_mean[s] = end > begin ? (float)(s_part[0] / (double)(end - begin)) : 0.f;
}

// Mean of the per-response means over the non-empty responses; one workgroup.
__global__ __launch_bounds__(kLossThreads) void policy_loss_batch_mean(const float* __restrict__ seq_mean,
                                                                        const int64_t* __restrict__ offsets,
                                                                        int32_t n_seq, float* __restrict__ out) {
    __shared__ double s_sum[kLossThreads];
    __shared__ int32_t s_cnt[kLossThreads];
    double acc = 0.0;
    int32_t cnt = 0;
    for (int32_t s = threadIdx.x; s < n_seq; s += kLossThreads)
        if (offsets[s + 1] > offsets[s]) { acc += (double)seq_mean[s]; ++cnt; }
    s_sum[threadIdx.x] = acc;
    s_cnt[threadIdx.x] = cnt;
    __syncthreads();
    for (int stride = kLossThreads / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) {
            s_sum[threadIdx.x] += s_sum[threadIdx.x + stride];
            s_cnt[threadIdx.x] += s_cnt[threadIdx.x + stride];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = s_cnt[0] ? (float)(s_sum[0] / s_cnt[0]) : 0.f;
}

}  // namespace

extern "C" int roll_policy_loss(const float* logp_theta, const float* logp_old, const float* logp_prox,
                                const float* signal, const int64_t* seq_offsets, float* value_out,
                                float* grad_out, float* is_weight_out, float* seq_mean_out,
                                float* batch_mean_out, const roll_loss_desc* d, void* stream_v) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->kind < ROLL_LOSS_PPO || d->kind > ROLL_LOSS_TOPR) return roll::fail(ROLL_ERR_INVALID_ARG, "unknown objective %d", d->kind);
    if (d->num_seqs <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "num_seqs must be > 0");
    if (!logp_theta || !logp_old || !signal || !seq_offsets || !seq_mean_out || !batch_mean_out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (d->kind == ROLL_LOSS_DECOUPLED_PPO && !logp_prox)
        return roll::fail(ROLL_ERR_INVALID_ARG, "Decoupled PPO needs logp_prox");
    if (!(d->eps_low >= 0.f) || !(d->eps_high >= 0.f) || !(d->c > 0.f))
        return roll::fail(ROLL_ERR_INVALID_ARG, "eps_low, eps_high must be >= 0 and c > 0");
    LossParams p{d->kind, (double)d->eps_low, (double)d->eps_high, (double)d->c};
    hipStream_t stream = (hipStream_t)stream_v;
    policy_loss_rows<<<d->num_seqs, kLossThreads, 0, stream>>>(logp_theta, logp_old, logp_prox, signal, seq_offsets,
                                                              value_out, grad_out, is_weight_out, seq_mean_out, p);
    ROLL_HIP_CHECK(hipGetLastError());
    policy_loss_batch_mean<<<1, kLossThreads, 0, stream>>>(seq_mean_out, seq_offsets, d->num_seqs, batch_mean_out);
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}
