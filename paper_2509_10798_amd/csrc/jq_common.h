// Internal declarations shared by the HIP sources of libjq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "jq.h"

namespace jq {

constexpr int kKeyTile = 32;        // keys per MFMA tile (one 32x32 block column)
constexpr int kRowTile = 32;        // query rows per MFMA tile
constexpr int kMaxRowTiles = 4;     // query-row tiles one wave keeps in registers (128 rows)
constexpr int kHeadDim = 128;
constexpr int kScoreWaves = 4;      // waves per workgroup in the score kernels
constexpr int kHistBins = 2048;     // level-1 radix bins (top 11 bits of the sortable key)
constexpr int kHistStride = kHistBins + 16;  // per problem: the bins, then [0] #sure and [1] #candidate counters
constexpr int kSelectThreads = 1024;
constexpr int kSegLen = 1024;       // positions per pooling workgroup = entries per segment of the selection's sorted lists

// Per-call sequence table, passed to kernels by value (about 2 KiB of kernarg).
struct SeqTab {
    int32_t n_seq;
    int32_t cu_seq[JQ_MAX_SEQ + 1];    // token offsets
    int32_t cu_bud[JQ_MAX_SEQ + 1];    // kept-row offsets
    int32_t cu_chunk[JQ_MAX_SEQ + 1];  // score-wave offsets (ceil(L / chunk_keys) waves per sequence and head)
    int32_t cu_cgrp[JQ_MAX_SEQ + 1];   // score-workgroup offsets (ceil(waves / 4) workgroups per sequence and head)
};

// Where a layer's K / V rows live: dense [T] rows per layer (block_table null), or a pool of n_pages pages of
// 1 << page_shift rows per layer with a per-sequence block table.
struct PageMap {
    const int32_t* block_table;  // DEVICE [n_seq][max_pages], or null
    int32_t page_shift, n_pages, max_pages;
};

// Everything the host derives from a jq_shape.
struct Plan {
    int32_t n_layers, n_seq, n_q, h_q, h_kv, d, group, pool_k;
    int32_t keep_first, keep_last;  // positions at either end of a sequence that the selection always keeps
    int32_t window;                 // 1: the queries are the last n_q tokens of every sequence (causal inside them)
    const int32_t* layer_budgets;   // DEVICE [n_layers][n_seq] or null: per-layer budgets (tab.cu_bud then holds the largest)
    int32_t rows;         // n_q * group: query rows that share one KV head
    int32_t row_tiles;    // ceil(rows / 32)
    int32_t row_groups;   // ceil(row_tiles / 4): passes of the score kernels over K
    int32_t chunk_keys;   // a sequence of L keys gets ceil(L / chunk_keys) score waves per head (multiple of 32)
    int32_t n_chunks;     // such waves per layer and head, over all sequences (tab.cu_chunk counts them)
    // the same for the second K pass when a first one has run (tab holds the first pass's tables)
    int32_t chunk_keys2, n_chunks2;
    int32_t cu_chunk2[JQ_MAX_SEQ + 1], cu_cgrp2[JQ_MAX_SEQ + 1];
    float scale;          // logit scale actually used
    // paged cache (block_table null: dense K, V): page = 1 << page_shift tokens, n_pages per layer's pool
    const int32_t* block_table;  // DEVICE [n_seq][max_pages]
    int32_t page_shift, n_pages, max_pages;
    int64_t T, TB;
    SeqTab tab;
    // pooling workgroups ("segments") per layer and head: ceil(L_s / kSegLen) per sequence, never across sequences
    int32_t n_seg;
    int32_t cu_seg[JQ_MAX_SEQ + 1];
    int32_t seg_head;  // entries kept per segment: several times the average kept positions per kSegLen scores
    PageMap page_map() const { return PageMap{block_table, page_shift, n_pages, max_pages}; }
    PageMap out_map;      // where the pruned cache goes (block_table null: dense [n_layers][TB] rows)
    void* const* marks;   // host only: nullptr, or 2 * kTraceKernels events (start, stop) for jq_evict_traced
    // workspace layout (byte offsets, 256-aligned)
    size_t off_stats, off_aug, off_hist, off_scores, off_pooled, off_idx, off_seg, off_seghdr, ws_bytes;
};

// Largest s with cu[s] <= v (cu[0] = 0, strictly increasing, v < cu[n]).
__host__ __device__ inline int find_seq(const int32_t* cu, int n, int64_t v) {
    int lo = 0, hi = n;  // answer in [lo, hi)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((int64_t)cu[mid] <= v) lo = mid; else hi = mid;
    }
    return lo;
}

// Order-preserving map from fp32 to uint32 (larger float <=> larger key); -0 is folded onto +0.
__device__ inline uint32_t sortable_key(float x) {
    uint32_t b = __float_as_uint(x + 0.0f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// A block-table entry as every kernel uses it: entries outside the pool (a corrupt table, the -1 of an unused slot)
// are clamped into it, so that the scored keys and the gathered rows always come from the same page.
__host__ __device__ inline int32_t clamp_page(int32_t entry, int32_t n_pages) {
    return entry < 0 ? 0 : (entry > n_pages - 1 ? n_pages - 1 : entry);
}

// Row (in units of token rows, over all layers) of token `pos` of sequence `s`; `cu` holds the sequences' dense
// offsets (token offsets for the cache, kept-row offsets for the pruned cache) and T their total.
__device__ inline int64_t kv_row(const PageMap& pm, const int32_t* cu, int64_t T, int layer, int s, int pos) {
    if (!pm.block_table) return (int64_t)layer * T + cu[s] + pos;
    const int32_t e = pm.block_table[(int64_t)s * pm.max_pages + (pos >> pm.page_shift)];
    const int64_t page = (int64_t)layer * pm.n_pages + clamp_page(e, pm.n_pages);
    return (page << pm.page_shift) + (pos & ((1 << pm.page_shift) - 1));
}

// In-place eviction: is the row that holds token `pos` of sequence `s` (row `src_row` of its layer when dense)
// among the rows the call overwrites?  Dense: the front TB rows of the layer.  Paged into the input's own pool:
// any row of a page that the output table names (`dest_bits`: one bit per page of the pool).
__device__ inline bool row_is_overwritten(const PageMap& pm, const uint32_t* dest_bits, int64_t src_row_dense, int64_t TB, int s,
                                          int pos) {
    if (!pm.block_table) return src_row_dense < TB;
    const int32_t e = clamp_page(pm.block_table[(int64_t)s * pm.max_pages + (pos >> pm.page_shift)], pm.n_pages);
    return (dest_bits[e >> 5] >> (e & 31)) & 1u;
}

// The same with the sequence's first dense row (`cu[s]` of kv_row) already looked up.
__device__ inline int64_t kv_row_from(const PageMap& pm, int64_t seq_row0, int64_t T, int layer, int s, int pos) {
    if (!pm.block_table) return (int64_t)layer * T + seq_row0 + pos;
    const int32_t e = pm.block_table[(int64_t)s * pm.max_pages + (pos >> pm.page_shift)];
    const int64_t page = (int64_t)layer * pm.n_pages + clamp_page(e, pm.n_pages);
    return (page << pm.page_shift) + (pos & ((1 << pm.page_shift) - 1));
}

// Budget of (layer, sequence): the table's segment length, or the caller's per-layer value clamped into
// max(1, forced) .. that, where `forced` = keep_first + keep_last is the number of positions that are kept whatever
// they score (the host has checked forced <= segment length; it cannot see the per-layer values).
__device__ inline uint32_t budget_of(const int32_t* layer_budgets, const SeqTab& tab, int layer, int s, int forced) {
    const int32_t cap = tab.cu_bud[s + 1] - tab.cu_bud[s];
    if (!layer_budgets) return (uint32_t)cap;
    return (uint32_t)min(max(layer_budgets[(int64_t)layer * tab.n_seq + s], max(forced, 1)), cap);
}

// Key the top-B selection ranks position j of an L-token sequence by: always-kept positions outrank
// every score.
__device__ inline uint32_t select_key(float x, int j, int L, int keep_first, int keep_last) {
    return (j < keep_first || j >= L - keep_last) ? 0xFFFFFFFFu : sortable_key(x);
}

// Ablation and diagnosis knobs, read from the environment ONCE per process (first use) -- no entry point touches the
// environment on its hot path.  jq_reload_knobs() reads them again (tests use it to force rarely taken paths).
struct Knobs {
    int32_t chunk_keys;   // JQ_CHUNK_KEYS: keys per wave in the pass that reads K cold (0: planned from the call's size)
    int32_t chunk_keys2;  // JQ_CHUNK_KEYS_2: the same for the second pass (0: JQ_CHUNK_KEYS if set, else planned)
    int32_t depth1, depth2;  // JQ_DEPTH_1 / JQ_DEPTH_2: key tiles a wave keeps in flight (1 or 2)
    int32_t log;          // JQ_LOG: print the HIP error string when a launch is refused
};
const Knobs& knobs();

// Stores of a kernel's bulk OUTPUT (pooled scores, block heads, kept positions and rows): nothing in the same
// kernel reads them back, the next kernel does.  Left in L2 as dirty lines they are written back when the kernel
// ends, and the next kernel cannot start before that: the gap between two dependent kernels grows with what the
// first one wrote (2.45 / 2.98 / 3.32 us after 4 / 16 / 64 MB, whatever the second kernel's shape).  Stored
// non-temporally they are on their way out while the kernel still runs.  Measured with the builds side by side in
// one process: kept rows -1.1 us per step (the next step's first kernel starts sooner), pooling's outputs -0.4 us
// more; for the second pass's scores it makes no difference, so they stay plain stores.  Agent-scope stores (sc1)
// did the same for pooling and nothing for the kept rows.
typedef uint32_t jq_u32x4 __attribute__((ext_vector_type(4)));
template <class T>
__device__ __forceinline__ void store_stream(T* p, T v) {  // T: float or int32_t
    __builtin_nontemporal_store(v, p);
}
__device__ __forceinline__ void store_stream16(void* p, uint4 v) {
    const jq_u32x4 x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, (jq_u32x4*)p);
}

// Workgroup barrier that orders LDS traffic only: global loads and stores that are still outstanding stay in
// flight across it (a plain __syncthreads() waits for all of them first).  For workgroups that communicate
// through LDS alone.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Inclusive prefix sum over a block of THREADS threads (thread order); `tmp` (LDS) holds THREADS/64 + 1 words.
template <int THREADS>
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t* tmp, uint32_t* total) {
    constexpr int kW = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    lds_barrier();  // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = x;
    lds_barrier();
    if (wave == 0) {
        const uint32_t w = lane < kW ? tmp[lane] : 0u;
        uint32_t wi = w;
#pragma unroll
        for (int d = 1; d < kW; d <<= 1) {
            const uint32_t y = __shfl_up(wi, d);
            if (lane >= d) wi += y;
        }
        if (lane < kW) tmp[lane] = wi - w;  // exclusive wave offsets
        if (lane == kW - 1) tmp[kW] = wi;
    }
    lds_barrier();
    *total = tmp[kW];
    return x + tmp[wave];
}

// Kernels whose start/stop timestamps jq_evict_traced reports, in launch order.
enum TraceKernel { kTrStats = 0, kTrScore, kTrPool, kTrFinalize, kTraceKernels };

// Launch through hipLaunchKernel so that the status belongs to this launch alone (the sticky
// "last error" of the runtime may hold an unrelated, earlier code from the host application).
// With `marks` set, the launch carries the (start, stop) events of slot `tr`, which receive the
// dispatch's own begin/end timestamps.
template <typename Kernel, typename... Args>
inline hipError_t launch_kernel(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                                void* const* marks, int tr, Args... args) {
    void* ptrs[] = {(void*)&args...};
    if (marks && tr >= 0)
        return hipExtLaunchKernel((const void*)kernel, grid, block, ptrs, lds_bytes, st, (hipEvent_t)marks[2 * tr],
                                  (hipEvent_t)marks[2 * tr + 1], 0);
    return hipLaunchKernel((const void*)kernel, grid, block, ptrs, lds_bytes, st);
}

// Stage launchers (enqueue only).  Each returns a hipError_t from the launch.
// `zero_words` words at `zero` (nullable) are cleared on the way (between the two K passes).
// With `lse` (nullable, [n_layers, n_seq, n_q, h_q] natural-log normalisers) the statistics pass is skipped.
// With `k_tail` (nullable, [n_layers, n_seq, n_q, h_kv, d] bf16) the normalisers also cover those keys, causally.
// With `fuse` the last launch of the second pass does not store its scores: it compares them with a reference
// map and leaves one partial sum of squared differences per workgroup (Eq. 5 forward, see launch_mse_reduce).
struct MseFuse {
    const float* ref;         // [n_layers][h_kv][T] scores of the other query set
    float inv_rows_ref, inv_rows_own;
    double* part;             // [n_layers][workgroups of the second pass per layer and head][h_kv]
};
hipError_t launch_score(const Plan& p, const void* Q, const void* K, float* scores, char* ws, hipStream_t st,
                        uint32_t* zero = nullptr, size_t zero_words = 0, const float* lse = nullptr,
                        const void* k_tail = nullptr, const MseFuse* fuse = nullptr);
// Sums the per-workgroup partials of a fused launch in workgroup order and divides by the sequence length.
hipError_t launch_mse_reduce(const Plan& p, const double* part, float* mse, hipStream_t st);
// With `hist` the pooling kernel also builds the selection's level-1 histograms, and with `ws` on top of that
// the per-workgroup sorted lists (segments) that the selection's fast path reads.
hipError_t launch_pool(const Plan& p, const float* scores, float* pooled, uint32_t* hist_or_null, char* ws_or_null,
                       hipStream_t st);
hipError_t launch_map_mse(const Plan& p, const float* scores_a, float rows_a, const float* scores_b, float rows_b,
                          float* mse, hipStream_t st);
hipError_t launch_fill_u32(uint32_t* dst, size_t n, uint32_t v, hipStream_t st);
hipError_t launch_hist(const Plan& p, const float* pooled, uint32_t* hist, char* ws_or_null, hipStream_t st);
// Whether every sequence of the plan fits the selection's fast path (LDS bitmaps); otherwise it streams.
bool select_fast_path(const Plan& p);
// With K, V, K_out, V_out (all or none) the selection also gathers the kept rows when its fast path runs;
// `*gathered` tells whether it did (otherwise launch_compact is still due).  With K, V and `stage` (in-place
// eviction, dense layouts, no K_out / V_out) it copies the kept rows whose sources are about to be overwritten to
// `stage` instead; launch_compact_inplace_write then finishes the job (`*gathered` false: the full
// launch_compact_inplace is due).  With pos_in / pos_out (streaming eviction: [n_layers][h_kv][T] and
// [n_layers][h_kv][TB]) every kept row's entry of pos_in is written next to its position.
hipError_t launch_select(const Plan& p, const float* pooled, uint32_t* hist, char* ws, int32_t* idx, hipStream_t st,
                         const void* K = nullptr, const void* V = nullptr, void* K_out = nullptr, void* V_out = nullptr,
                         bool* gathered = nullptr, void* stage = nullptr, const int32_t* pos_in = nullptr,
                         int32_t* pos_out = nullptr, const uint32_t* dest_bits = nullptr);
hipError_t launch_compact(const Plan& p, const void* K, const void* V, const int32_t* idx, void* K_out, void* V_out,
                          hipStream_t st);
// In place: kept rows land at the front of K / V themselves; `stage` holds 2 * n_layers * TB * h_kv rows.
hipError_t launch_compact_inplace(const Plan& p, void* K, void* V, const int32_t* idx, void* stage, hipStream_t st,
                                  const uint32_t* dest_bits = nullptr);
// Only its second launch: every kept row written, from `stage` (rows staged earlier) or from its untouched source.
// With paged K / V (p.block_table) the kept rows go where p.out_map says, inside the same pools; `dest_bits` then
// marks the pages that receive rows (one bit per page; null for the dense layout).
hipError_t launch_compact_inplace_write(const Plan& p, void* K, void* V, const int32_t* idx, void* stage, hipStream_t st,
                                        const uint32_t* dest_bits = nullptr);
// Bitmap of the pages that p.out_map's table names for kept rows (one launch; ceil(n_pages / 32) words).
hipError_t launch_mark_dest_pages(const Plan& p, uint32_t* dest_bits, hipStream_t st);

// `cu_ref_budgets`: n_seq + 1 prefix sums of the reference list lengths, `tb_ref` their total.
hipError_t launch_hit_rate(const Plan& p, const int32_t* cu_ref_budgets, int64_t tb_ref, const int32_t* cur,
                           const int32_t* ref, float* rate, hipStream_t st);
hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st);

}  // namespace jq
