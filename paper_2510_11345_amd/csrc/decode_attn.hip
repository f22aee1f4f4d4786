// Paged GQA decode attention for gfx950: work-list build, split-K partial
// attention on the matrix cores, LDS-staged merge across the waves of a
// workgroup, and a second-stage merge across chunks.
//
// ROLL Flash (arXiv 2510.11345) Section 1: decoding is memory-bandwidth bound
// and response lengths are long-tailed; Section 4.2: one step over the whole
// running batch per loop iteration.  The kernel's only job is therefore to
// stream each live KV byte exactly once at HBM speed while rows of very
// different lengths share the chip evenly.
//
// Work decomposition.  Row b with L_b tokens is cut into ceil(L_b / C) chunks
// of C tokens; one workgroup of kWaves wavefronts handles one (row, chunk, KV
// head) unit, wave w taking the 32-token steps w, w + kWaves, ...  All G = Hq /
// Hkv query heads that share the KV head ride in one MFMA tile, so a KV byte
// is fetched once and used G times.
//
// Per 32-token step and wave (lane = 16 * q + r):
//   S^T[tok][g]  = K[tok][:] . Q[g][:]      2 tiles x (D/32) v_mfma_f32_16x16x32_bf16,
//                  K rows as the A operand (16 bytes per lane straight from the page),
//                  Q as the B operand (held in registers for the whole unit);
//   online softmax per head g = r over the 8 scores a lane owns (tokens 8q..8q+7),
//                  one cross-lane max over q per step;
//   O^T[d][g]   += V^T[d][tok] . P^T[tok][g]  (D/16) x 2 MFMAs, V octets as the A operand,
//                  P split into a bf16 high part and a bf16 remainder as two B operands so
//                  that the probabilities keep ~16 mantissa bits (the fp32-output tolerance
//                  does not survive an 8-bit P).
// The accumulator layout of S^T (a lane owns 4 consecutive token rows of a tile for one
// head) is exactly the B-operand layout of the PV product once the two S tiles are laid
// side by side, so P never moves between lanes.  Which 8 tokens a lane owns is free as
// long as K rows and V octets agree: tile tt, row 4*q'+i  <->  token 8*q' + 4*tt + i.
#include <cfloat>
#include <cmath>

#include "common.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int kWaves = 4;          // wavefronts per workgroup
constexpr bool kPipeline = false;   // issue the next step's loads before computing the current one
constexpr int kStep = 32;          // tokens per wave step
constexpr int kDefaultChunk = 512; // tokens per split-K chunk
constexpr int kCounterInts = 64;   // 256-byte header of the workspace

struct AttnParams {
    int32_t B, Hq, Hkv, G;
    int32_t log2P, max_pages, num_pages;
    int32_t chunk_tokens, max_len;
    int32_t max_chunks;  // capacity of the work list and of the partial buffers
    int32_t out_f32;
    float scale_log2e;
};

struct Workspace {
    int32_t* counters;       // [0] = number of chunks
    int32_t* chunk_offsets;  // [B + 1] exclusive prefix of chunks per row
    int2* work;              // [max_chunks] (row, chunk index in row)
    float2* part_ml;         // [max_chunks * Hq] (max in log2 units, sum)
    float* part_acc;         // [max_chunks * Hq * D] un-normalised output
    size_t bytes;
    int64_t max_chunks;
};

__host__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

__host__ Workspace carve(void* base, int32_t B, int32_t Hq, int32_t D, int32_t chunk, int64_t max_len,
                         int64_t max_total) {
    Workspace w{};
    const int64_t per_row = (max_len + chunk - 1) / chunk;
    int64_t max_chunks = (int64_t)B * per_row;
    if (max_total > 0) max_chunks = std::min<int64_t>(max_chunks, max_total / chunk + B);
    if (max_chunks < 1) max_chunks = 1;
    w.max_chunks = max_chunks;
    size_t off = 0;
    char* p = (char*)base;
    w.counters = (int32_t*)(p + off);       off = align_up(off + sizeof(int32_t) * kCounterInts, 256);
    w.chunk_offsets = (int32_t*)(p + off);  off = align_up(off + sizeof(int32_t) * ((size_t)B + 1), 256);
    w.work = (int2*)(p + off);              off = align_up(off + sizeof(int2) * (size_t)max_chunks, 256);
    w.part_ml = (float2*)(p + off);         off = align_up(off + sizeof(float2) * (size_t)max_chunks * Hq, 256);
    w.part_acc = (float*)(p + off);         off = align_up(off + sizeof(float) * (size_t)max_chunks * Hq * D, 256);
    w.bytes = off;
    return w;
}

// ---------------------------------------------------------------------------
// Work list: chunks per row, exclusive prefix sum, flat (row, chunk) list.
// One workgroup; rows are scanned in tiles of blockDim.x.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void build_worklist(const int32_t* __restrict__ seq_lens,
                                                        int32_t B, int32_t chunk, int32_t max_len,
                                                        int64_t max_chunks,
                                                        int32_t* __restrict__ counters,
                                                        int32_t* __restrict__ chunk_offsets,
                                                        int2* __restrict__ work) {
    __shared__ int32_t s_scan[1024];
    __shared__ int32_t s_carry;
    const int tid = threadIdx.x;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int32_t base = 0; base < B; base += blockDim.x) {
        const int32_t b = base + tid;
        int32_t n = 0;
        if (b < B) {
            int32_t L = seq_lens[b];
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
            n = (L + chunk - 1) / chunk;
        }
        s_scan[tid] = n;
        __syncthreads();
        for (int off = 1; off < (int)blockDim.x; off <<= 1) {
            int32_t v = tid >= off ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        const int32_t carry = s_carry;
        const int32_t incl = s_scan[tid] + carry;
        const int32_t excl = incl - n;
        if (b < B) {
            chunk_offsets[b] = excl;
            for (int32_t c = 0; c < n; ++c)
                if ((int64_t)excl + c < max_chunks) work[excl + c] = make_int2(b, c);
        }
        __syncthreads();
        if (tid == (int)blockDim.x - 1) s_carry = incl;
        __syncthreads();
    }
    if (tid == 0) {
        const int32_t total = s_carry;
        chunk_offsets[B] = total;
        counters[0] = (int64_t)total < max_chunks ? total : (int32_t)max_chunks;
    }
}

// ---------------------------------------------------------------------------
// Split-K partial attention.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// KV is read exactly once per step: a nontemporal load keeps it from displacing the
// page table, Q and the partials in L2 (measured: +10 % on a plain streaming read).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    f32x2_t f = {lo, hi};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

template <int D>
struct StepData {
    uint4 k[2][D / 32];
    uint4 v[D / 16];
};

template <int D>
struct WaveCtx {
    const uint4* __restrict__ k_pages;
    const uint4* __restrict__ v_pages;
    const int32_t* __restrict__ pt_row;
    int32_t h, Hkv, log2P, num_pages, max_pages, r, q;
};

template <int D>
__device__ __forceinline__ void load_step(const WaveCtx<D>& c, int32_t t0, StepData<D>& s) {
    const int32_t P = 1 << c.log2P;
    int32_t pa = t0 >> c.log2P;
    // The second page may lie past the row's end; its table entry is then stale or -1.  Reading
    // it is in bounds (clamped to the table row) and the id is clamped below, so the loads stay
    // inside the pool; the tokens are masked by the caller.  Not clamping to the row's own
    // last page keeps the row length off the address path.
    int32_t pb = (t0 + 16) >> c.log2P;
    pb = pb > c.max_pages - 1 ? c.max_pages - 1 : pb;
    int32_t pgA = c.pt_row[pa];
    int32_t pgB = c.pt_row[pb];
    pgA = pgA < 0 ? 0 : (pgA >= c.num_pages ? c.num_pages - 1 : pgA);
    pgB = pgB < 0 ? 0 : (pgB >= c.num_pages ? c.num_pages - 1 : pgB);
    // K: lane (r, q) reads, for tile tt and k-block kk, 8 head-dim elements 32kk+8q.. of
    // token 8*(r>>2) + 4*tt + (r&3).
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int32_t tis = 8 * (c.r >> 2) + 4 * tt + (c.r & 3);
        const int32_t page = tis >= 16 ? pgB : pgA;
        const int32_t tin = (t0 + tis) & (P - 1);
        const uint4* base = c.k_pages + (((int64_t)page * c.Hkv + c.h) * (D / 8) + c.q) * P + tin;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) s.k[tt][kk] = load_stream(base + (int64_t)kk * 4 * P);
    }
    // V: lane (r, q) reads, for d-tile nt, the 8 tokens 8q..8q+7 of head-dim element 16nt+r.
    {
        const int32_t page = c.q >= 2 ? pgB : pgA;
        const int32_t oct = ((t0 + 8 * c.q) & (P - 1)) >> 3;
        const uint4* base = c.v_pages + (((int64_t)page * c.Hkv + c.h) * (P / 8) + oct) * D + c.r;
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) s.v[nt] = load_stream(base + nt * 16);
    }
}

template <int D>
struct WaveAcc {
    f32x4_t o[D / 16];  // O^T tiles: lane (r, q) holds head r, head-dim 16nt + 4q + i
    float m;            // running max of head r, log2 units
    float l;            // this lane's share of the running sum of head r
};

template <int D>
__device__ __forceinline__ void compute_step(const WaveCtx<D>& c, const bf16x8_t (&qf)[D / 32],
                                             StepData<D>& s, int32_t t0, int32_t end,
                                             float scale_log2e, WaveAcc<D>& a) {
    f32x4_t sc[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s.k[tt][kk]), qf[kk], acc, 0, 0, 0);
        sc[tt] = acc;
    }
    float sv[8];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[4 * tt + i] = sc[tt][i] * scale_log2e;

    if (t0 + kStep > end) {  // ragged tail of the row: mask scores and zero the V octets
        const int32_t first = t0 + 8 * c.q;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (first + j >= end) sv[j] = -INFINITY;
        const int32_t nvalid = end - first;
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

    float mx = sv[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(a.m, mx);   // finite: every processed step has a valid token
    const float alpha = __builtin_amdgcn_exp2f(a.m - m_new);
    a.m = m_new;
    float p[8];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(sv[j] - m_new);
        psum += p[j];
    }
    a.l = a.l * alpha + psum;

    uint32_t hi[4], lo[4];
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
        hi[k2] = pack_bf16_rne(p[2 * k2], p[2 * k2 + 1]);
        const float r0 = p[2 * k2] - __uint_as_float(hi[k2] << 16);
        const float r1 = p[2 * k2 + 1] - __uint_as_float(hi[k2] & 0xFFFF0000u);
        lo[k2] = pack_bf16_rne(r0, r1);
    }
    const bf16x8_t p_hi = as_bf16x8(make_uint4(hi[0], hi[1], hi[2], hi[3]));
    const bf16x8_t p_lo = as_bf16x8(make_uint4(lo[0], lo[1], lo[2], lo[3]));

    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) a.o[nt] *= alpha;
    }
#pragma unroll
    for (int nt = 0; nt < D / 16; ++nt) {
        const bf16x8_t vf = as_bf16x8(s.v[nt]);
        a.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, p_hi, a.o[nt], 0, 0, 0);
        a.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, p_lo, a.o[nt], 0, 0, 0);
    }
}

template <int D, bool PIPE>
__global__ __launch_bounds__(kWaves * 64) void attn_partial(
    const uint4* __restrict__ q16, const uint4* __restrict__ k_pages, const uint4* __restrict__ v_pages,
    const int32_t* __restrict__ page_table, const int32_t* __restrict__ seq_lens,
    const int2* __restrict__ work, const int32_t* __restrict__ counters,
    const int32_t* __restrict__ chunk_offsets, void* __restrict__ out, float2* __restrict__ part_ml,
    float* __restrict__ part_acc, AttnParams prm) {
    extern __shared__ float smem[];
    const int32_t total_units = counters[0] * prm.Hkv;
    const int32_t unit = blockIdx.x;
    if (unit >= total_units) return;
    const int2 entry = work[unit / prm.Hkv];
    const int32_t h = unit % prm.Hkv;
    const int32_t b = entry.x, ci = entry.y;
    int32_t L = seq_lens[b];
    L = L < 0 ? 0 : (L > prm.max_len ? prm.max_len : L);
    const int32_t start = ci * prm.chunk_tokens;
    const int32_t end = min(L, start + prm.chunk_tokens);
    const int32_t n_steps = (end - start + kStep - 1) / kStep;
    const int32_t row_chunk0 = chunk_offsets[b];
    const int32_t n_chunks = chunk_offsets[b + 1] - row_chunk0;

    const int32_t lane = threadIdx.x & 63;
    const int32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t G = prm.G;

    WaveCtx<D> ctx;
    ctx.k_pages = k_pages;
    ctx.v_pages = v_pages;
    ctx.pt_row = page_table + (int64_t)b * prm.max_pages;
    ctx.h = h;
    ctx.Hkv = prm.Hkv;
    ctx.log2P = prm.log2P;
    ctx.num_pages = prm.num_pages;
    ctx.max_pages = prm.max_pages;
    ctx.r = lane & 15;
    ctx.q = lane >> 4;

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

    if (PIPE) {
        StepData<D> s0, s1;
        int32_t s = wave;
        if (s < n_steps) {
            load_step<D>(ctx, start + s * kStep, s0);
            for (;;) {
                const int32_t sn = s + kWaves;
                const bool has1 = sn < n_steps;
                if (has1) load_step<D>(ctx, start + sn * kStep, s1);
                compute_step<D>(ctx, qf, s0, start + s * kStep, end, prm.scale_log2e, acc);
                if (!has1) break;
                s = sn + kWaves;
                const bool has0 = s < n_steps;
                if (has0) load_step<D>(ctx, start + s * kStep, s0);
                compute_step<D>(ctx, qf, s1, start + sn * kStep, end, prm.scale_log2e, acc);
                if (!has0) break;
            }
        }
    } else {
        for (int32_t s = wave; s < n_steps; s += kWaves) {
            StepData<D> sd;
            load_step<D>(ctx, start + s * kStep, sd);
            compute_step<D>(ctx, qf, sd, start + s * kStep, end, prm.scale_log2e, acc);
        }
    }

    // Finish the per-head sum across the four q-groups of the wave.
    acc.l += __shfl_xor(acc.l, 16);
    acc.l += __shfl_xor(acc.l, 32);

    // LDS-staged merge across the waves of the workgroup.
    const int32_t ldo = D + 4;                           // padded row of the O staging tile
    float* s_m = smem;                                   // [kWaves][16]
    float* s_l = smem + kWaves * 16;                     // [kWaves][16]
    float* s_o = smem + 2 * kWaves * 16;                 // [kWaves][G][ldo]
    if (ctx.q == 0) {
        s_m[wave * 16 + ctx.r] = acc.m;
        s_l[wave * 16 + ctx.r] = acc.l;
    }
    if (ctx.r < G) {
        float* dst = s_o + ((int64_t)(wave * G + ctx.r)) * ldo + 4 * ctx.q;
#pragma unroll
        for (int nt = 0; nt < D / 16; ++nt) *(f32x4_t*)(dst + 16 * nt) = acc.o[nt];
    }
    __syncthreads();

    const int32_t chunk_global = row_chunk0 + ci;
    for (int32_t e = threadIdx.x; e < G * D; e += kWaves * 64) {
        const int32_t g = e / D, d = e % D;
        float M = s_m[g];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w * 16 + g]);
        float lsum = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = __builtin_amdgcn_exp2f(s_m[w * 16 + g] - M);  // 0 for an idle wave
            lsum += s_l[w * 16 + g] * wgt;
            o += s_o[(w * G + g) * ldo + d] * wgt;
        }
        const int32_t head = h * G + g;
        if (n_chunks == 1) {
            const float val = o / lsum;
            const int64_t idx = ((int64_t)b * prm.Hq + head) * D + d;
            if (prm.out_f32) ((float*)out)[idx] = val;
            else ((__bf16*)out)[idx] = (__bf16)val;
        } else {
            const int64_t ph = (int64_t)chunk_global * prm.Hq + head;
            part_acc[ph * D + d] = o;
            if (d == 0) part_ml[ph] = make_float2(M, lsum);
        }
    }
}

// ---------------------------------------------------------------------------
// Second-stage merge across the chunks of a row; also zero-fills empty rows.
// One workgroup per (row, KV head); a thread owns (head, d) outputs.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_merge(const int32_t* __restrict__ seq_lens,
                                                   const int32_t* __restrict__ chunk_offsets,
                                                   const float2* __restrict__ part_ml,
                                                   const float* __restrict__ part_acc,
                                                   void* __restrict__ out, int32_t D, AttnParams prm) {
    const int32_t b = blockIdx.x / prm.Hkv;
    const int32_t h = blockIdx.x % prm.Hkv;
    const int32_t c0 = chunk_offsets[b];
    const int32_t n_all = chunk_offsets[b + 1] - c0;
    if (n_all == 1) return;
    // Chunks past the capacity were never computed (the caller's max_total_tokens was too low).
    const int32_t n = c0 + n_all <= prm.max_chunks ? n_all : (c0 < prm.max_chunks ? prm.max_chunks - c0 : 0);
    const int32_t G = prm.G;
    for (int32_t e = threadIdx.x; e < G * D; e += blockDim.x) {
        const int32_t g = e / D, d = e % D;
        const int32_t head = h * G + g;
        float val = 0.f;
        if (n > 1) {
            float M = -INFINITY;
            for (int32_t c = 0; c < n; ++c) M = fmaxf(M, part_ml[(int64_t)(c0 + c) * prm.Hq + head].x);
            float lsum = 0.f, o = 0.f;
            for (int32_t c = 0; c < n; ++c) {
                const int64_t ph = (int64_t)(c0 + c) * prm.Hq + head;
                const float2 ml = part_ml[ph];
                const float wgt = __builtin_amdgcn_exp2f(ml.x - M);
                lsum += ml.y * wgt;
                o += part_acc[ph * D + d] * wgt;
            }
            val = o / lsum;
        }
        const int64_t idx = ((int64_t)b * prm.Hq + head) * D + d;
        if (prm.out_f32) ((float*)out)[idx] = val;
        else ((__bf16*)out)[idx] = (__bf16)val;
    }
}

int validate(const roll_attn_desc* d) {
    if (!d) return roll::fail(ROLL_ERR_INVALID_ARG, "desc is NULL");
    if (d->batch <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "batch must be > 0");
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads != 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "num_q_heads must be a positive multiple of num_kv_heads");
    if (d->num_q_heads / d->num_kv_heads > 16)
        return roll::fail(ROLL_ERR_INVALID_ARG, "GQA group size above 16 is not supported");
    if (d->head_dim != 64 && d->head_dim != 128) return roll::fail(ROLL_ERR_INVALID_ARG, "head_dim must be 64 or 128");
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64");
    if (d->max_pages_per_seq <= 0 || d->num_pages <= 0) return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq and num_pages must be > 0");
    if ((int64_t)d->max_pages_per_seq * d->page_size > (1 << 30))
        return roll::fail(ROLL_ERR_INVALID_ARG, "max_pages_per_seq * page_size above 2^30 tokens");
    if (d->out_dtype != ROLL_BF16 && d->out_dtype != ROLL_F32) return roll::fail(ROLL_ERR_INVALID_ARG, "out_dtype must be ROLL_BF16 or ROLL_F32");
    if (d->chunk_tokens < 0 || d->chunk_tokens % (kWaves * kStep) != 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "chunk_tokens must be 0 or a multiple of %d", kWaves * kStep);
    if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return roll::fail(ROLL_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    if (d->max_total_tokens < 0) return roll::fail(ROLL_ERR_INVALID_ARG, "max_total_tokens < 0");
    return ROLL_OK;
}

}  // namespace

extern "C" size_t roll_decode_attn_workspace_bytes(const roll_attn_desc* d) {
    if (validate(d) != ROLL_OK) return 0;
    const int32_t chunk = d->chunk_tokens ? d->chunk_tokens : kDefaultChunk;
    return carve(nullptr, d->batch, d->num_q_heads, d->head_dim, chunk,
                 (int64_t)d->max_pages_per_seq * d->page_size, d->max_total_tokens).bytes;
}

extern "C" int roll_decode_attn(const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* page_table, const int32_t* seq_lens, void* out,
                                const roll_attn_desc* d, void* workspace, size_t workspace_bytes,
                                void* stream_v) {
    int rc = validate(d);
    if (rc != ROLL_OK) return rc;
    if (!q || !k_pages || !v_pages || !page_table || !seq_lens || !out)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(q, 16) || !roll::aligned(k_pages, 16) || !roll::aligned(v_pages, 16) || !roll::aligned(out, 16) ||
        !roll::aligned(page_table, 4) || !roll::aligned(seq_lens, 4))
        return roll::fail(ROLL_ERR_INVALID_ARG, "q, k_pages, v_pages, out must be 16-byte aligned");
    const int32_t chunk = d->chunk_tokens ? d->chunk_tokens : kDefaultChunk;
    const int64_t max_len = (int64_t)d->max_pages_per_seq * d->page_size;
    if (!workspace || !roll::aligned(workspace, 256)) return roll::fail(ROLL_ERR_WORKSPACE, "workspace NULL or not 256-byte aligned");
    Workspace ws = carve(workspace, d->batch, d->num_q_heads, d->head_dim, chunk, max_len, d->max_total_tokens);
    if (workspace_bytes < ws.bytes)
        return roll::fail(ROLL_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, ws.bytes);
    if (ws.max_chunks * d->num_kv_heads * 2 > INT32_MAX) return roll::fail(ROLL_ERR_INVALID_ARG, "too many work units");

    hipStream_t stream = (hipStream_t)stream_v;
    AttnParams prm{};
    prm.B = d->batch;
    prm.Hq = d->num_q_heads;
    prm.Hkv = d->num_kv_heads;
    prm.G = d->num_q_heads / d->num_kv_heads;
    prm.log2P = d->page_size == 16 ? 4 : (d->page_size == 32 ? 5 : 6);
    prm.max_pages = d->max_pages_per_seq;
    prm.num_pages = d->num_pages;
    prm.chunk_tokens = chunk;
    prm.max_len = (int32_t)max_len;
    prm.max_chunks = (int32_t)ws.max_chunks;
    prm.out_f32 = d->out_dtype == ROLL_F32;
    const float scale = d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / sqrtf((float)d->head_dim);
    prm.scale_log2e = scale * 1.44269504088896340736f;

    build_worklist<<<1, 1024, 0, stream>>>(seq_lens, d->batch, chunk, prm.max_len, ws.max_chunks,
                                           ws.counters, ws.chunk_offsets, ws.work);
    ROLL_HIP_CHECK(hipGetLastError());

    const unsigned grid = (unsigned)(ws.max_chunks * d->num_kv_heads);
    const size_t lds = sizeof(float) * (2 * kWaves * 16 + (size_t)kWaves * prm.G * (d->head_dim + 4));
    if (d->ev_main_begin) ROLL_HIP_CHECK(hipEventRecord((hipEvent_t)d->ev_main_begin, stream));
    if (d->head_dim == 128)
        attn_partial<128, kPipeline><<<grid, kWaves * 64, lds, stream>>>(
            (const uint4*)q, (const uint4*)k_pages, (const uint4*)v_pages, page_table, seq_lens, ws.work,
            ws.counters, ws.chunk_offsets, out, ws.part_ml, ws.part_acc, prm);
    else
        attn_partial<64, kPipeline><<<grid, kWaves * 64, lds, stream>>>(
            (const uint4*)q, (const uint4*)k_pages, (const uint4*)v_pages, page_table, seq_lens, ws.work,
            ws.counters, ws.chunk_offsets, out, ws.part_ml, ws.part_acc, prm);
    ROLL_HIP_CHECK(hipGetLastError());
    if (d->ev_main_end) ROLL_HIP_CHECK(hipEventRecord((hipEvent_t)d->ev_main_end, stream));

    attn_merge<<<d->batch * d->num_kv_heads, 256, 0, stream>>>(seq_lens, ws.chunk_offsets, ws.part_ml,
                                                              ws.part_acc, out, d->head_dim, prm);
    ROLL_HIP_CHECK(hipGetLastError());
    return ROLL_OK;
}
