// Pruned KV cache (paper Section 4.3: decoding continues on the pruned cache): gather the kept
// rows of K and V into dense [TB, h_kv, d] tensors.  Pure copy, 16 bytes per lane, 16 lanes per
// 256-byte head row; consecutive lanes/waves write consecutive output bytes.
#include "jq_common.h"

namespace jq {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct CompactArgs {
    const char* K; const char* V;
    char* K_out; char* V_out;
    const int32_t* idx;  // [n_layers][h_kv][TB], sequence-local
    int32_t n_layers, h_kv;
    int64_t T, TB;
    PageMap pm;      // where the rows of K and V live (dense or paged)
    PageMap pm_out;  // where the kept rows go
    const int32_t* layer_budgets;  // DEVICE [n_layers][n_seq] or null: slots beyond a layer's own budget are skipped
    int32_t forced;                // keep_first + keep_last: the least a per-layer budget can be
    SeqTab tab;
};

constexpr int kCompactThreads = 256;
constexpr int kLanesPerRow = kHeadDim * 2 / 16;  // 16

__global__ __launch_bounds__(kCompactThreads) void jq_compact_kernel(CompactArgs a) {
    // item = (layer, kept row tb, head g), g fastest: the output is written front to back
    const int64_t n_items = (int64_t)a.n_layers * a.TB * a.h_kv;
    const int64_t item = ((int64_t)blockIdx.x * kCompactThreads + threadIdx.x) / kLanesPerRow;
    if (item >= n_items) return;
    const int part = threadIdx.x % kLanesPerRow;
    const int g = (int)(item % a.h_kv);
    const int64_t rest = item / a.h_kv;
    const int64_t tb = rest % a.TB;
    const int layer = (int)(rest / a.TB);
    const int s = find_seq(a.tab.cu_bud, a.tab.n_seq, tb);
    const int L = a.tab.cu_seq[s + 1] - a.tab.cu_seq[s];
    if ((uint32_t)(tb - a.tab.cu_bud[s]) >= budget_of(a.layer_budgets, a.tab, layer, s, a.forced)) return;
    int j = a.idx[((int64_t)layer * a.h_kv + g) * a.TB + tb];
    j = min(max(j, 0), L - 1);  // never read outside the sequence
    const int64_t src = ((kv_row(a.pm, a.tab.cu_seq, a.T, layer, s, j) * a.h_kv + g) * kHeadDim) * 2 + part * 16;
    const int64_t dst = ((kv_row(a.pm_out, a.tab.cu_bud, a.TB, layer, s, (int)(tb - a.tab.cu_bud[s])) * a.h_kv + g) * kHeadDim) * 2 + part * 16;
    const u32x4 kv = *(const u32x4*)(a.K + src);
    const u32x4 vv = *(const u32x4*)(a.V + src);
    __builtin_nontemporal_store(kv, (u32x4*)(a.K_out + dst));  // bulk output: see store_stream()
    __builtin_nontemporal_store(vv, (u32x4*)(a.V_out + dst));
}

hipError_t launch_compact(const Plan& p, const void* K, const void* V, const int32_t* idx, void* K_out, void* V_out,
                          hipStream_t st) {
    CompactArgs a;
    a.K = (const char*)K; a.V = (const char*)V; a.K_out = (char*)K_out; a.V_out = (char*)V_out;
    a.idx = idx;
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.T = p.T; a.TB = p.TB;
    a.pm = p.page_map();
    a.pm_out = p.out_map;
    a.layer_budgets = p.layer_budgets;
    a.forced = p.keep_first + p.keep_last;
    a.tab = p.tab;
    const int64_t threads = (int64_t)p.n_layers * p.TB * p.h_kv * kLanesPerRow;
    return launch_kernel(jq_compact_kernel, dim3((unsigned)((threads + kCompactThreads - 1) / kCompactThreads)),
                         dim3(kCompactThreads), 0, st, nullptr, -1, a);
}

// In-place variant: the kept rows of a layer land in rows 0..TB-1 of that layer's own K / V.  A kept row
// whose source is one of those rows could be overwritten by another workgroup before it is read, so such
// rows go through a staging buffer: launch 1 copies them out, launch 2 writes every kept row, taking it from
// the staging buffer or from its (never overwritten) source beyond the front.
struct InplaceArgs {
    char* K; char* V;
    char* stage;         // [2][n_layers][TB][h_kv][d] bf16: K rows, then V rows
    const int32_t* idx;  // [n_layers][h_kv][TB], sequence-local
    const uint32_t* dest_bits;  // paged: one bit per page of the pool, set for pages that receive kept rows
    PageMap pm, pm_out;         // paged: where the rows live / where the kept rows go (same pools); dense: no tables
    int32_t n_layers, h_kv;
    int64_t T, TB;
    const int32_t* layer_budgets;  // DEVICE [n_layers][n_seq] or null
    int32_t forced;                // keep_first + keep_last: the least a per-layer budget can be
    SeqTab tab;
};

template <bool WRITE>
__global__ __launch_bounds__(kCompactThreads) void jq_compact_inplace_kernel(InplaceArgs a) {
    const int64_t n_items = (int64_t)a.n_layers * a.TB * a.h_kv;
    const int64_t item = ((int64_t)blockIdx.x * kCompactThreads + threadIdx.x) / kLanesPerRow;
    if (item >= n_items) return;
    const int part = threadIdx.x % kLanesPerRow;
    const int g = (int)(item % a.h_kv);
    const int64_t rest = item / a.h_kv;
    const int64_t tb = rest % a.TB;
    const int layer = (int)(rest / a.TB);
    const int s = find_seq(a.tab.cu_bud, a.tab.n_seq, tb);
    const int L = a.tab.cu_seq[s + 1] - a.tab.cu_seq[s];
    if ((uint32_t)(tb - a.tab.cu_bud[s]) >= budget_of(a.layer_budgets, a.tab, layer, s, a.forced)) return;  // slot not used by this layer
    int j = a.idx[((int64_t)layer * a.h_kv + g) * a.TB + tb];
    j = min(max(j, 0), L - 1);
    const int64_t src_row = (int64_t)a.tab.cu_seq[s] + j;  // within the layer (dense layout)
    const bool staged = row_is_overwritten(a.pm, a.dest_bits, src_row, a.TB, s, j);  // the source is a row that this call overwrites
    const int64_t src = ((kv_row(a.pm, a.tab.cu_seq, a.T, layer, s, j) * a.h_kv + g) * kHeadDim) * 2 + part * 16;
    const int64_t stg = item * (kHeadDim * 2) + part * 16;
    const int64_t v_stage = n_items * (kHeadDim * 2);
    if (!WRITE) {
        if (!staged) return;
        *(u32x4*)(a.stage + stg) = *(const u32x4*)(a.K + src);
        *(u32x4*)(a.stage + v_stage + stg) = *(const u32x4*)(a.V + src);
    } else {
        // dense: row tb of the layer's own K / V; paged: where the output table puts kept row tb - cu_bud[s]
        const int64_t dst_row = a.pm_out.block_table ? kv_row(a.pm_out, a.tab.cu_bud, a.TB, layer, s, (int)(tb - a.tab.cu_bud[s]))
                                                     : (int64_t)layer * a.T + tb;
        const int64_t dst = ((dst_row * a.h_kv + g) * kHeadDim) * 2 + part * 16;
        const u32x4 kv = staged ? *(const u32x4*)(a.stage + stg) : *(const u32x4*)(a.K + src);
        const u32x4 vv = staged ? *(const u32x4*)(a.stage + v_stage + stg) : *(const u32x4*)(a.V + src);
        __builtin_nontemporal_store(kv, (u32x4*)(a.K + dst));  // bulk output: see store_stream()
        __builtin_nontemporal_store(vv, (u32x4*)(a.V + dst));
    }
}

static InplaceArgs inplace_args(const Plan& p, void* K, void* V, const int32_t* idx, void* stage, dim3* grid,
                                const uint32_t* dest_bits = nullptr) {
    InplaceArgs a;
    a.K = (char*)K; a.V = (char*)V; a.stage = (char*)stage; a.idx = idx;
    a.dest_bits = dest_bits;
    a.pm = p.page_map();
    a.pm_out = p.out_map;
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.T = p.T; a.TB = p.TB;
    a.layer_budgets = p.layer_budgets;
    a.forced = p.keep_first + p.keep_last;
    a.tab = p.tab;
    const int64_t threads = (int64_t)p.n_layers * p.TB * p.h_kv * kLanesPerRow;
    *grid = dim3((unsigned)((threads + kCompactThreads - 1) / kCompactThreads));
    return a;
}

hipError_t launch_compact_inplace(const Plan& p, void* K, void* V, const int32_t* idx, void* stage, hipStream_t st,
                                  const uint32_t* dest_bits) {
    dim3 grid;
    const InplaceArgs a = inplace_args(p, K, V, idx, stage, &grid, dest_bits);
    hipError_t e = launch_kernel(jq_compact_inplace_kernel<false>, grid, dim3(kCompactThreads), 0, st, nullptr, -1, a);
    if (e != hipSuccess) return e;
    return launch_kernel(jq_compact_inplace_kernel<true>, grid, dim3(kCompactThreads), 0, st, nullptr, -1, a);
}

hipError_t launch_compact_inplace_write(const Plan& p, void* K, void* V, const int32_t* idx, void* stage, hipStream_t st,
                                        const uint32_t* dest_bits) {
    dim3 grid;
    const InplaceArgs a = inplace_args(p, K, V, idx, stage, &grid, dest_bits);
    return launch_kernel(jq_compact_inplace_kernel<true>, grid, dim3(kCompactThreads), 0, st, nullptr, -1, a);
}

// One workgroup: clear the bitmap, then set the bit of every page that the output table names for a kept row.
struct MarkArgs {
    uint32_t* bits;
    PageMap out;       // the output table
    int32_t n_words;   // ceil(n_pages / 32)
    SeqTab tab;        // cu_bud: kept rows per sequence
};
__global__ __launch_bounds__(1024) void jq_mark_dest_pages_kernel(MarkArgs a) {
    for (int w = threadIdx.x; w < a.n_words; w += 1024) a.bits[w] = 0u;
    __syncthreads();
    for (int s = 0; s < a.tab.n_seq; ++s) {
        const int B = a.tab.cu_bud[s + 1] - a.tab.cu_bud[s];
        const int n = (B + (1 << a.out.page_shift) - 1) >> a.out.page_shift;  // pages of sequence s that receive rows
        for (int j = threadIdx.x; j < n; j += 1024) {
            const int32_t e = clamp_page(a.out.block_table[(int64_t)s * a.out.max_pages + j], a.out.n_pages);
            atomicOr(&a.bits[e >> 5], 1u << (e & 31));
        }
    }
}

hipError_t launch_mark_dest_pages(const Plan& p, uint32_t* dest_bits, hipStream_t st) {
    MarkArgs a;
    a.bits = dest_bits;
    a.out = p.out_map;
    a.n_words = (p.out_map.n_pages + 31) / 32;
    a.tab = p.tab;
    return launch_kernel(jq_mark_dest_pages_kernel, dim3(1), dim3(1024), 0, st, nullptr, -1, a);
}

// Critical-KV hit rate (paper Eq. 6): |I_cur & I_ref| / |I_ref| per (layer, sequence, KV head) for two kept
// sets given as ascending position lists.  One workgroup per problem; every position of the reference
// list is looked up in the current list by binary search.  Integer work; the quotient is the only rounding.
struct HitArgs {
    const int32_t* cur;  // [n_layers][h_kv][TB_cur]
    const int32_t* ref;  // [n_layers][h_kv][TB_ref]
    float* rate;         // [n_layers][n_seq][h_kv]
    int32_t n_layers, n_seq, h_kv;
    int64_t TB_cur, TB_ref;
    int32_t cu_cur[JQ_MAX_SEQ + 1], cu_ref[JQ_MAX_SEQ + 1];
};

__global__ __launch_bounds__(256) void jq_hit_rate_kernel(HitArgs a) {
    __shared__ uint32_t wave_hits[4];
    const int g = blockIdx.x % a.h_kv;
    const int s = (blockIdx.x / a.h_kv) % a.n_seq;
    const int layer = blockIdx.x / (a.h_kv * a.n_seq);
    const int nc = a.cu_cur[s + 1] - a.cu_cur[s], nr = a.cu_ref[s + 1] - a.cu_ref[s];
    const int32_t* cur = a.cur + ((int64_t)layer * a.h_kv + g) * a.TB_cur + a.cu_cur[s];
    const int32_t* ref = a.ref + ((int64_t)layer * a.h_kv + g) * a.TB_ref + a.cu_ref[s];
    uint32_t hits = 0;
    for (int i = threadIdx.x; i < nr; i += 256) {
        const int32_t want = ref[i];
        int lo = 0, hi = nc;  // first position of cur that is >= want
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (cur[mid] < want) lo = mid + 1; else hi = mid;
        }
        hits += (lo < nc && cur[lo] == want);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) hits += __shfl_xor(hits, d);
    if ((threadIdx.x & 63) == 0) wave_hits[threadIdx.x >> 6] = hits;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t total = wave_hits[0] + wave_hits[1] + wave_hits[2] + wave_hits[3];
        a.rate[((int64_t)layer * a.n_seq + s) * a.h_kv + g] = (float)total / (float)nr;
    }
}

hipError_t launch_hit_rate(const Plan& p, const int32_t* cu_ref_budgets, int64_t tb_ref, const int32_t* cur,
                           const int32_t* ref, float* rate, hipStream_t st) {
    HitArgs a;
    a.cur = cur; a.ref = ref; a.rate = rate;
    a.n_layers = p.n_layers; a.n_seq = p.n_seq; a.h_kv = p.h_kv;
    a.TB_cur = p.TB; a.TB_ref = tb_ref;
    for (int s = 0; s <= p.n_seq; ++s) { a.cu_cur[s] = p.tab.cu_bud[s]; a.cu_ref[s] = cu_ref_budgets[s]; }
    return launch_kernel(jq_hit_rate_kernel, dim3((unsigned)(p.n_layers * p.n_seq * p.h_kv)), dim3(256), 0, st, nullptr, -1, a);
}

// Plain streaming copy, 16 bytes per lane: the known-size reference against which hardware traffic
// counters are calibrated.
__global__ __launch_bounds__(256) void jq_copy_probe_kernel(const u32x4* src, u32x4* dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256 * 64 ? want : 256 * 64);
    return launch_kernel(jq_copy_probe_kernel, dim3(blocks), dim3(256), 0, st, nullptr, -1, (const u32x4*)src, (u32x4*)dst,
                         n16);
}

}  // namespace jq
