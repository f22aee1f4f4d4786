// The per-step arithmetic shared by the decode and the prefill attention kernels (device code).
//
// One step is 32 KV tokens against 16 "columns" (decode: the query heads of one KV head;
// prefill: 16 query tokens of one head) on v_mfma_f32_16x16x32_bf16, lane = 16 * q + r:
//   S^T[tok][col] = K[tok][:] . Q[col][:]      2 tiles x (D/32) MFMAs, K rows as the A operand,
//                   Q as the B operand (held in registers);
//   online softmax per column r over the 8 scores a lane owns (tokens 8q..8q+7 of the step),
//                   one cross-lane max over q per step;
//   O^T[d][col]  += V^T[d][tok] . P^T[tok][col]  (D/16) x 2 MFMAs, V octets as the A operand,
//                   P split into a bf16 high part and a bf16 remainder as two B operands so
//                   that the probabilities keep ~16 mantissa bits.
// The accumulator layout of S^T (a lane owns 4 consecutive token rows of a tile for one
// column) is exactly the B-operand layout of the PV product once the two S tiles are laid
// side by side, so P never moves between lanes.  Which 8 tokens a lane owns is free as long
// as K rows and V octets agree: tile tt, row 4*q'+i  <->  token 8*q' + 4*tt + i.
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

namespace roll {
namespace attn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int kStep = 32;  // tokens per step

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    f32x2_t f = {lo, hi};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

// The MFMA A operands of one step.  k[tt][kk]: lane (r, q) holds head-dim 32kk + 8q .. + 7 of
// token 8*(r>>2) + 4*tt + (r&3) of the step.  v[nt]: lane (r, q) holds the tokens 8q .. 8q+7 of
// head-dim element 16nt + r.
template <int D>
struct StepData {
    uint4 k[2][D / 32];
    uint4 v[D / 16];
};

template <int D>
struct WaveAcc {
    f32x4_t o[D / 16];  // O^T tiles: lane (r, q) holds column r, head-dim 16nt + 4q + i
    float m;            // running max of column r, log2 units
    float l;            // this lane's share of the running sum of column r
};

// Maximum / sum over the four lanes that share a column (lanes r, r + 16, r + 32, r + 48), in
// every one of them.  v_permlane16_swap exchanges the odd 16-lane rows of its first operand
// with the even rows of its second, v_permlane32_swap the upper half of the first with the
// lower half of the second; with the same value in both operands the two results of a swap
// are the value of the lane itself and that of its partner (in either order), so combining
// them is the xor-16 (xor-32) step of a butterfly, without a trip through LDS.
__device__ __forceinline__ float max_over_q(float v) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float sum_over_q(float v) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Raw scores q . k of the step's 32 tokens for column r; the 8 a lane owns are the step's
// tokens 8q + j.  No scaling, no masking.
template <int D>
__device__ __forceinline__ void qk_scores_of(const bf16x8_t (&qf)[D / 32], const uint4 (&k)[2][D / 32], float (&sv)[8]) {
    f32x4_t sc[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k[tt][kk]), qf[kk], acc, 0, 0, 0);
        sc[tt] = acc;
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[4 * tt + i] = sc[tt][i];
}
template <int D>
__device__ __forceinline__ void qk_scores(const bf16x8_t (&qf)[D / 32], const StepData<D>& s, float (&sv)[8]) {
    qk_scores_of<D>(qf, s.k, sv);
}

// Zero the V elements of this lane's tokens nvalid, nvalid + 1, .. 7 (tokens that do not exist
// may hold anything, and 0 * NaN is NaN).
template <int D>
__device__ __forceinline__ void mask_v_tail(StepData<D>& s, int32_t nvalid) {
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        uint32_t w[4] = {s.v[nt].x, s.v[nt].y, s.v[nt].z, s.v[nt].w};
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
            const uint32_t keep = (2 * k2 < nvalid ? 0x0000FFFFu : 0u) | (2 * k2 + 1 < nvalid ? 0xFFFF0000u : 0u);
            w[k2] &= keep;
        }
        s.v[nt] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Online softmax update with the step's raw scores (-inf = masked; the running max must be
// finite afterwards) and O^T += V^T P^T.  scale_log2e = softmax scale * log2(e) > 0 is applied
// inside the exponent's fused multiply-add; the running max is kept in log2 units.  SPLIT: P as a bf16 high part plus a bf16 remainder (two
// MFMAs per tile); without it P is rounded to bf16 once, which is enough for a bf16 result.
// The probabilities of one step as the B operands of the PV product, and the factor by which
// the running sums shrink.
struct StepProbs {
    bf16x8_t hi, lo;   // lo is unused without SPLIT
    float alpha;
};

// First half of the update: running max and sum, probabilities.  Straight-line code.
template <bool SPLIT>
__device__ __forceinline__ StepProbs softmax_probs(const float (&sv)[8], float scale_log2e, float& m, float& l) {
    float mx = sv[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
    mx = max_over_q(mx) * scale_log2e;
    const float m_new = fmaxf(m, mx);
    StepProbs out;
    out.alpha = __builtin_amdgcn_exp2f(m - m_new);
    m = m_new;
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(fmaf(sv[j], scale_log2e, -m_new));
        psum += p[j];
    }
    l = l * out.alpha + psum;

    uint32_t hi[4], lo[4];
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
        hi[k2] = pack_bf16_rne(p[2 * k2], p[2 * k2 + 1]);
        if (SPLIT) {
            const float r0 = p[2 * k2] - __uint_as_float(hi[k2] << 16);
            const float r1 = p[2 * k2 + 1] - __uint_as_float(hi[k2] & 0xFFFF0000u);
            lo[k2] = pack_bf16_rne(r0, r1);
        } else {
            lo[k2] = 0u;
        }
    }
    out.hi = as_bf16x8(make_uint4(hi[0], hi[1], hi[2], hi[3]));
    out.lo = as_bf16x8(make_uint4(lo[0], lo[1], lo[2], lo[3]));
    return out;
}

// The update with a lazily moved reference, for kernels bound by vector work: as long as no
// score of the step exceeds the running reference a.m by more than kLazyBits (log2 units) the
// reference stays, no maximum is taken and nothing is rescaled; probabilities may then be as
// large as 2^kLazyBits, which neither bf16 nor the fp32 sums mind, and the final division by
// l makes the result the same.  When some lane of the wave does exceed it (always in a row's
// first step, where a.m is -inf), the reference moves to the exact running maximum, the sums are
// rescaled, and the exponents are taken again: at most one such round per call.
constexpr float kLazyBits = 8.0f;
template <int D, bool SPLIT>
__device__ __forceinline__ StepProbs softmax_probs_lazy(const float (&sv)[8], float scale_log2e, WaveAcc<D>& a) {
    float t[8];
#pragma unroll
    for (int round = 0; round < 2; ++round) {
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = fmaf(sv[j], scale_log2e, -a.m);
        const float top = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
        if (round == 1 || !__any(!(top <= kLazyBits))) break;
        float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
        mx = max_over_q(mx) * scale_log2e;
        const float m_new = fmaxf(a.m, mx);
        const float alpha = __builtin_amdgcn_exp2f(a.m - m_new);
        a.m = m_new;
        a.l *= alpha;
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) a.o[nt] *= alpha;
    }
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(t[j]);
        psum += p[j];
    }
    a.l += psum;
    StepProbs out;
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
        hi[k2] = pack_bf16_rne(p[2 * k2], p[2 * k2 + 1]);
        if (SPLIT) {
            const float r0 = p[2 * k2] - __uint_as_float(hi[k2] << 16);
            const float r1 = p[2 * k2 + 1] - __uint_as_float(hi[k2] & 0xFFFF0000u);
            lo[k2] = pack_bf16_rne(r0, r1);
        } else {
            lo[k2] = 0u;
        }
    }
    out.hi = as_bf16x8(make_uint4(hi[0], hi[1], hi[2], hi[3]));
    out.lo = as_bf16x8(make_uint4(lo[0], lo[1], lo[2], lo[3]));
    out.alpha = 1.0f;
    return out;
}

// Parts of the update on their own, for a kernel that overlaps them with other work.
// move_reference: the reference of the columns goes to the exact running maximum including this
// step's scores, sums and O^T are rescaled.
template <int D>
__device__ __forceinline__ void move_reference(const float (&sv)[8], float scale_log2e, WaveAcc<D>& a) {
    float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    mx = max_over_q(mx) * scale_log2e;
    const float m_new = fmaxf(a.m, mx);
    const float alpha = __builtin_amdgcn_exp2f(a.m - m_new);
    a.m = m_new;
    a.l *= alpha;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) a.o[nt] *= alpha;
}
// Probabilities as PV operands: rounded to bf16 once, or (SPLIT) as a bf16 high part plus a bf16
// remainder.
template <bool SPLIT>
__device__ __forceinline__ StepProbs pack_probs(const float (&p)[8]) {
    StepProbs out;
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
        hi[k2] = pack_bf16_rne(p[2 * k2], p[2 * k2 + 1]);
        if (SPLIT) {
            const float r0 = p[2 * k2] - __uint_as_float(hi[k2] << 16);
            const float r1 = p[2 * k2 + 1] - __uint_as_float(hi[k2] & 0xFFFF0000u);
            lo[k2] = pack_bf16_rne(r0, r1);
        } else {
            lo[k2] = 0u;
        }
    }
    out.hi = as_bf16x8(make_uint4(hi[0], hi[1], hi[2], hi[3]));
    out.lo = as_bf16x8(make_uint4(lo[0], lo[1], lo[2], lo[3]));
    out.alpha = 1.0f;
    return out;
}
// Second half: O^T = alpha O^T (skipped by the caller's test when no lane needs it) + V^T P^T.
template <int D>
__device__ __forceinline__ void rescale(WaveAcc<D>& a, float alpha) {
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) a.o[nt] *= alpha;
}
template <int D, bool SPLIT>
__device__ __forceinline__ void pv_accumulate(const StepData<D>& s, const StepProbs& pr, WaveAcc<D>& a) {
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        const bf16x8_t vf = as_bf16x8(s.v[nt]);
        a.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pr.hi, a.o[nt], 0, 0, 0);
        if (SPLIT) a.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pr.lo, a.o[nt], 0, 0, 0);
    }
}

template <int D, bool SPLIT = true>
__device__ __forceinline__ void softmax_pv(const float (&sv)[8], const StepData<D>& s, float scale_log2e,
                                           WaveAcc<D>& a) {
    const StepProbs pr = softmax_probs<SPLIT>(sv, scale_log2e, a.m, a.l);
    if (__any(pr.alpha != 1.0f)) rescale<D>(a, pr.alpha);
    pv_accumulate<D, SPLIT>(s, pr, a);
}

// Write one head-dim quad row of a finished column: normalise by the sum and store at
// out[idx + 16nt .. + 3] (elements of out_f32 ? float : bf16).
template <int D>
__device__ __forceinline__ void store_result(const WaveAcc<D>& a, void* __restrict__ out, int64_t idx,
                                             int32_t out_f32) {
    const float inv = 1.0f / a.l;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        const f32x4_t o = a.o[nt] * inv;
        if (out_f32) {
            *(f32x4_t*)((float*)out + idx + 16 * nt) = o;
        } else {
            uint2 pk;
            pk.x = pack_bf16_rne(o[0], o[1]);
            pk.y = pack_bf16_rne(o[2], o[3]);
            *(uint2*)((__bf16*)out + idx + 16 * nt) = pk;
        }
    }
}

// The same with the output type fixed at compile time.
template <int D, bool F32>
__device__ __forceinline__ void store_result_as(const WaveAcc<D>& a, void* __restrict__ out, int64_t idx) {
    const float inv = 1.0f / a.l;
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        const f32x4_t o = a.o[nt] * inv;
        if (F32) {
            *(f32x4_t*)((float*)out + idx + 16 * nt) = o;
        } else {
            uint2 pk;
            pk.x = pack_bf16_rne(o[0], o[1]);
            pk.y = pack_bf16_rne(o[2], o[3]);
            *(uint2*)((__bf16*)out + idx + 16 * nt) = pk;
        }
    }
}

}  // namespace attn
}  // namespace roll
