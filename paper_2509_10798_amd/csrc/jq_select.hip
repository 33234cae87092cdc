// Top-B retention per (layer, sequence, KV head) -- "retain the key-value pairs corresponding to
// the top-k highest scores" (paper Section 4.3) -- as an exact three-level radix select on the
// order-preserving 32-bit key of the pooled fp32 score, followed by an ordered compaction.
//
//   level 1: bits 31..21 (histogram supplied by the pooling kernel)   -> bin b1
//   level 2: bits 20..10 of the elements in b1                         -> bin b2
//   level 3: bits  9..0  of the elements in (b1, b2)                   -> threshold key tau
//   final:   keep key > tau, plus the first (B - #greater) positions with key == tau, writing
//            positions in ascending order (block-wide prefix sums over position order).
//
// One workgroup of 1024 threads per problem; the score row is streamed from L2 three times.
#include "jq_common.h"

namespace jq {

struct SelectArgs {
    const float* pooled;   // [n_layers][h_kv][T]
    const uint32_t* hist;  // [n_layers][n_seq][h_kv][kHistBins]
    int32_t* idx;          // [n_layers][h_kv][TB]
    int32_t h_kv;
    int64_t T, TB;
    SeqTab tab;
};

constexpr int kWaves = kSelectThreads / 64;

// Inclusive prefix sum over the block (thread order); `tmp` holds kWaves + 1 words.
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t v, uint32_t* tmp, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();  // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    if (wave == 0) {
        uint32_t w = lane < kWaves ? tmp[lane] : 0u;
        uint32_t wi = w;
#pragma unroll
        for (int d = 1; d < kWaves; d <<= 1) {
            const uint32_t y = __shfl_up(wi, d);
            if (lane >= d) wi += y;
        }
        if (lane < kWaves) tmp[lane] = wi - w;  // exclusive wave offsets
        if (lane == kWaves - 1) tmp[kWaves] = wi;
    }
    __syncthreads();
    *total = tmp[kWaves];
    return x + tmp[wave];
}

// Given bins[0..n_bins) (LDS), find the bin b such that (#elements in bins > b) < need <=
// (#elements in bins >= b).  Returns b and writes that count of strictly greater elements.
// n_bins must be a multiple of kSelectThreads or smaller; uses two bins per thread at most.
__device__ __forceinline__ uint32_t pick_bin(const uint32_t* bins, int n_bins, uint32_t need, uint32_t* tmp,
                                             uint32_t* result /* LDS: [0]=bin, [1]=above */) {
    // thread t owns the bins (n_bins-1-2t) and (n_bins-2-2t): descending order
    const int b_hi = n_bins - 1 - 2 * (int)threadIdx.x, b_lo = b_hi - 1;
    const uint32_t c_hi = b_hi >= 0 ? bins[b_hi] : 0u;
    const uint32_t c_lo = b_lo >= 0 ? bins[b_lo] : 0u;
    uint32_t total;
    const uint32_t incl = block_scan_incl(c_hi + c_lo, tmp, &total);
    const uint32_t before = incl - (c_hi + c_lo);  // elements in bins above b_hi
    if (before < need && need <= before + c_hi) { result[0] = (uint32_t)b_hi; result[1] = before; }
    else if (before + c_hi < need && need <= incl) { result[0] = (uint32_t)b_lo; result[1] = before + c_hi; }
    __syncthreads();
    return result[0];
}

__global__ __launch_bounds__(kSelectThreads) void jq_select_kernel(SelectArgs a) {
    __shared__ uint32_t bins[kHistBins];
    __shared__ uint32_t tmp[kWaves + 1];
    __shared__ uint32_t res[2];

    const int prob = blockIdx.x;
    const int g = prob % a.h_kv;
    const int s = (prob / a.h_kv) % a.tab.n_seq;
    const int layer = prob / (a.h_kv * a.tab.n_seq);
    const int L = a.tab.cu_seq[s + 1] - a.tab.cu_seq[s];
    const uint32_t B = (uint32_t)(a.tab.cu_bud[s + 1] - a.tab.cu_bud[s]);
    const float* x = a.pooled + ((int64_t)layer * a.h_kv + g) * a.T + a.tab.cu_seq[s];
    int32_t* out = a.idx + ((int64_t)layer * a.h_kv + g) * a.TB + a.tab.cu_bud[s];
    const uint32_t* h1 = a.hist + (((int64_t)layer * a.tab.n_seq + s) * a.h_kv + g) * kHistBins;

    // ---- level 1 -----------------------------------------------------------------------------
    for (int b = threadIdx.x; b < kHistBins; b += kSelectThreads) bins[b] = h1[b];
    __syncthreads();
    uint32_t need = B;
    const uint32_t b1 = pick_bin(bins, kHistBins, need, tmp, res);
    need -= res[1];
    __syncthreads();

    // ---- level 2 -----------------------------------------------------------------------------
    for (int b = threadIdx.x; b < kHistBins; b += kSelectThreads) bins[b] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < L; j += kSelectThreads) {
        const uint32_t k = sortable_key(x[j]);
        if ((k >> 21) == b1) atomicAdd(&bins[(k >> 10) & 2047u], 1u);
    }
    __syncthreads();
    const uint32_t b2 = pick_bin(bins, 2048, need, tmp, res);
    need -= res[1];
    __syncthreads();

    // ---- level 3 -----------------------------------------------------------------------------
    const uint32_t prefix22 = (b1 << 11) | b2;
    for (int b = threadIdx.x; b < 1024; b += kSelectThreads) bins[b] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < L; j += kSelectThreads) {
        const uint32_t k = sortable_key(x[j]);
        if ((k >> 10) == prefix22) atomicAdd(&bins[k & 1023u], 1u);
    }
    __syncthreads();
    const uint32_t b3 = pick_bin(bins, 1024, need, tmp, res);
    need -= res[1];  // how many elements equal to tau are kept
    __syncthreads();
    const uint32_t tau = (prefix22 << 10) | b3;

    // ---- ordered compaction ------------------------------------------------------------------
    // Each thread takes 4 consecutive positions per round, so thread order is position order.
    uint32_t gt_done = 0, eq_done = 0;  // kept-so-far counts before this round (uniform)
    for (int base = 0; base < L; base += kSelectThreads * 4) {
        const int j0 = base + threadIdx.x * 4;
        uint32_t kk[4];
        uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            kk[e] = (j0 + e < L) ? sortable_key(x[j0 + e]) : 0u;  // key 0 is below every real key
            n_gt += (j0 + e < L) && kk[e] > tau;
            n_eq += (j0 + e < L) && kk[e] == tau;
        }
        uint32_t total;
        const uint32_t packed = n_gt | (n_eq << 16);  // at most 4096 per field and round
        const uint32_t incl = block_scan_incl(packed, tmp, &total);
        uint32_t gt_before = gt_done + ((incl - packed) & 0xFFFFu);
        uint32_t eq_before = eq_done + ((incl - packed) >> 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (j0 + e >= L) break;
            const bool is_gt = kk[e] > tau, is_eq = kk[e] == tau;
            if (is_gt || (is_eq && eq_before < need)) {
                const uint32_t slot = gt_before + min(eq_before, need);
                if (slot < B) out[slot] = j0 + e;  // always true for consistent histograms; guards NaN-poisoned input
            }
            gt_before += is_gt;
            eq_before += is_eq;
        }
        gt_done += total & 0xFFFFu;
        eq_done += total >> 16;
        if (gt_done + min(eq_done, need) >= B) break;  // uniform: everything kept already
    }
}

hipError_t launch_select(const Plan& p, const float* pooled, const uint32_t* hist, int32_t* idx, hipStream_t st) {
    SelectArgs a;
    a.pooled = pooled; a.hist = hist; a.idx = idx;
    a.h_kv = p.h_kv; a.T = p.T; a.TB = p.TB;
    a.tab = p.tab;
    const unsigned n_prob = (unsigned)((int64_t)p.n_layers * p.n_seq * p.h_kv);
    return launch_kernel(jq_select_kernel, dim3(n_prob), dim3(kSelectThreads), st, a);
}

}  // namespace jq
