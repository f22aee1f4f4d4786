// Profiling helper: a plain streaming read of exactly the paged KV bytes a decode step reads,
// through the same page table, with no arithmetic on them.  What it reaches is the bandwidth
// this box gives to that access pattern (pages scattered over the pool, the K and the V block of
// a page each read once), the ceiling the attention kernel is to be compared with beside the
// published peak.
//
// ROLL Flash (arXiv 2510.11345) Section 1: decoding is memory-bandwidth bound; the measure of a
// decode-attention kernel is therefore how close it comes to what the memory system can deliver.
#include "common.h"

namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeMaxBatch = 8192;

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// One workgroup per (row, page) unit at a time, units taken grid-stride.  A unit is the K block
// and the V block of one page (all KV heads): blk16 16-byte pieces each.
__global__ __launch_bounds__(kProbeThreads) void kv_read_probe(
    const u32x4_t* __restrict__ k_pages, const u32x4_t* __restrict__ v_pages,
    const int32_t* __restrict__ page_table, const int32_t* __restrict__ seq_lens, int32_t B, int32_t log2P,
    int32_t max_pages, int32_t num_pages, int64_t stride16, int32_t blk16, uint32_t* __restrict__ sink) {
    __shared__ int32_t pre[kProbeMaxBatch + 1];  // pages of the rows before b
    __shared__ int32_t s_part[kProbeThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t P = 1 << log2P;
    int32_t carry = 0;
    for (int32_t base = 0; base < B; base += kProbeThreads) {
        const int32_t b = base + tid;
        int32_t n = 0;
        if (b < B) {
            int32_t L = seq_lens[b];
            L = L < 0 ? 0 : L;
            n = (L + P - 1) >> log2P;
            n = n > max_pages ? max_pages : n;
        }
        int32_t incl = n;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        if (lane == 63) s_part[wave] = incl;
        __syncthreads();
        int32_t before = carry;
        for (int w = 0; w < wave; ++w) before += s_part[w];
        for (int w = 0; w < kProbeThreads / 64; ++w) carry += s_part[w];
        if (b < B) pre[b] = before + incl - n;
        __syncthreads();
    }
    if (tid == 0) pre[B] = carry;
    __syncthreads();
    const int32_t units = pre[B];
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (int32_t u = blockIdx.x; u < units; u += gridDim.x) {
        int32_t lo = 0, hi = B;  // pre[lo] <= u < pre[hi]
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) >> 1;
            if (pre[mid] <= u) lo = mid; else hi = mid;
        }
        int32_t page = page_table[(int64_t)lo * max_pages + (u - pre[lo])];
        page = page < 0 ? 0 : (page >= num_pages ? num_pages - 1 : page);
        const u32x4_t* kb = k_pages + (int64_t)page * stride16;
        const u32x4_t* vb = v_pages + (int64_t)page * stride16;
        for (int32_t i = tid; i < blk16; i += 4 * kProbeThreads) {
            u32x4_t a[4], c[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int32_t at = i + j * kProbeThreads;
                const int32_t safe = at < blk16 ? at : i;
                a[j] = __builtin_nontemporal_load(kb + safe);
                c[j] = __builtin_nontemporal_load(vb + safe);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= a[j] ^ c[j];
        }
    }
    // one word per thread keeps the loads alive; the value means nothing
    sink[(size_t)blockIdx.x * kProbeThreads + tid] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

}  // namespace

extern "C" int roll_prof_kv_read_probe(const void* k_pages, const void* v_pages, const int32_t* page_table,
                                       const int32_t* seq_lens, const roll_attn_desc* d, void* sink,
                                       size_t sink_bytes, int64_t* bytes_read_out, void* stream) {
    if (!d || !k_pages || !v_pages || !page_table || !seq_lens || !sink)
        return roll::fail(ROLL_ERR_INVALID_ARG, "NULL pointer argument");
    if (!roll::aligned(k_pages, 16) || !roll::aligned(v_pages, 16) || !roll::aligned(sink, 4))
        return roll::fail(ROLL_ERR_INVALID_ARG, "k_pages, v_pages must be 16-byte aligned");
    if (d->batch <= 0 || d->batch > kProbeMaxBatch) return roll::fail(ROLL_ERR_INVALID_ARG, "batch must be in [1, %d]", kProbeMaxBatch);
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64)
        return roll::fail(ROLL_ERR_INVALID_ARG, "page_size must be 16, 32 or 64");
    if (d->num_kv_heads <= 0 || d->head_dim <= 0 || d->head_dim % 8 != 0 || d->max_pages_per_seq <= 0 || d->num_pages <= 0)
        return roll::fail(ROLL_ERR_INVALID_ARG, "bad shape");
    const int32_t Hs = roll::page_stride_heads(d->page_stride, d->num_kv_heads, d->page_size, d->head_dim);
    if (Hs == 0) return roll::fail(ROLL_ERR_INVALID_ARG, "page_stride must be 0 or a multiple of page_size * head_dim that holds all KV heads");
    int dev = 0, cus = 0;
    ROLL_HIP_CHECK(hipGetDevice(&dev));
    ROLL_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const unsigned grid = (unsigned)(cus > 0 ? cus : 256) * 8u;
    if (sink_bytes < (size_t)grid * kProbeThreads * 4)
        return roll::fail(ROLL_ERR_WORKSPACE, "sink too small: %zu < %zu bytes", sink_bytes, (size_t)grid * kProbeThreads * 4);
    const int64_t block_elems = (int64_t)d->num_kv_heads * d->page_size * d->head_dim;
    const int32_t log2P = d->page_size == 16 ? 4 : (d->page_size == 32 ? 5 : 6);
    kv_read_probe<<<grid, kProbeThreads, 0, (hipStream_t)stream>>>(
        (const u32x4_t*)k_pages, (const u32x4_t*)v_pages, page_table, seq_lens, d->batch, log2P, d->max_pages_per_seq,
        d->num_pages, (int64_t)Hs * d->page_size * d->head_dim / 8, (int32_t)(block_elems / 8), (uint32_t*)sink);
    ROLL_HIP_CHECK(hipGetLastError());
    if (bytes_read_out) *bytes_read_out = 2 * block_elems * 2;  // per page: K block + V block, bf16
    return ROLL_OK;
}
