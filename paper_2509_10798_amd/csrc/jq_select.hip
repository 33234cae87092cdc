// Top-B retention per (layer, sequence, KV head): the B best-scored key-value pairs stay, the rest is
// dropped (paper Section 4.3) -- as an exact radix select on the order-preserving 32-bit key of the
// pooled fp32 score.  Ties go to the lower position; output is ascending.
//
//   level 1: bits 31..21, histogram supplied by the pooling kernel                    -> bin b1
//   level 2: bits 20..10 of the elements in b1                                         -> bin b2
//   level 3: bits  9..0  of the elements in (b1, b2)                                   -> threshold key tau
//   result : every key > tau, plus the first (B - #greater) positions with key == tau
//
// Fast path (every sequence of the call fits the LDS bitmaps):
//   scatter  -- the whole GPU streams the scores once; positions above bin b1 go to a "sure"
//               list, (key, position) pairs inside b1 to a candidate list (block-aggregated
//               appends; the order between blocks is arbitrary);
//   finalize -- a workgroup resolves levels 2 and 3 on a problem's candidates in LDS, marks sure /
//               chosen positions in an L-bit LDS bitmap, trims the tie group to its lowest
//               positions and emits set bits in ascending order.  Several workgroups ("slices")
//               work on one problem: each repeats the (cheap, L2-resident) resolution and emits
//               its own range of output slots; in the fused eviction call it also gathers the K/V
//               rows of those slots, so the pruned cache needs no further kernel.
// General path (very long sequences): one workgroup per problem streams the row three times.
#include <atomic>

#include "jq_common.h"

namespace jq {

struct SelectArgs {
    const float* pooled;  // [n_layers][h_kv][T]
    uint32_t* hist;       // [n_layers][n_seq][h_kv][kHistStride]: level-1 bins, then the two list counters
    int32_t* sure;        // [n_layers][h_kv][TB]   positions above bin b1 (unordered)
    uint2* cand;          // [n_layers][h_kv][T]    (key, position) inside bin b1 (unordered)
    int32_t* idx;         // [n_layers][h_kv][TB]
    int32_t n_layers, h_kv;
    int32_t keep_first, keep_last;  // always-kept positions at either end of every sequence
    int64_t T, TB;
    // fused gather (all four null when the kept rows are not wanted): K,V [n_layers][T][h_kv][d] bf16,
    // K_out,V_out [n_layers][TB][h_kv][d]
    const char* K; const char* V;
    char* K_out; char* V_out;
    PageMap pm;      // where the rows of K and V live (dense or paged)
    PageMap pm_out;  // where the kept rows go
    const int32_t* layer_budgets;  // DEVICE [n_layers][n_seq] or null
    SeqTab tab;
};

// Inclusive prefix sum over a block of THREADS threads (thread order); `tmp` holds THREADS/64 + 1 words.
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
    __syncthreads();  // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
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
    __syncthreads();
    *total = tmp[kW];
    return x + tmp[wave];
}

// bins[0..n_bins): find the bin b with (#elements in bins > b) < need <= (#elements in bins >= b).
// Thread t owns PER consecutive bins, highest bins first.  result[0] = b, result[1] = #elements above,
// result[2] = #elements inside b.
template <int THREADS, int PER, typename BinPtr>
__device__ __forceinline__ void pick_bin(BinPtr bins, int n_bins, uint32_t need, uint32_t* tmp, uint32_t* result) {
    uint32_t c[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int b = n_bins - 1 - (PER * (int)threadIdx.x + e);
        c[e] = b >= 0 ? bins[b] : 0u;
        sum += c[e];
    }
    uint32_t total;
    const uint32_t incl = block_scan_incl<THREADS>(sum, tmp, &total);
    uint32_t before = incl - sum;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        if (before < need && need <= before + c[e]) {
            result[0] = (uint32_t)(n_bins - 1 - (PER * (int)threadIdx.x + e));
            result[1] = before;
            result[2] = c[e];
        }
        before += c[e];
    }
    __syncthreads();
}

struct Problem {
    int layer, s, g, L;
    uint32_t B;
    const float* x;
    int32_t* out;
    uint32_t* hist;
};

__device__ __forceinline__ Problem problem_of(const SelectArgs& a, int prob) {
    Problem p;
    p.g = prob % a.h_kv;
    p.s = (prob / a.h_kv) % a.tab.n_seq;
    p.layer = prob / (a.h_kv * a.tab.n_seq);
    p.L = a.tab.cu_seq[p.s + 1] - a.tab.cu_seq[p.s];
    p.B = budget_of(a.layer_budgets, a.tab, p.layer, p.s, a.keep_first + a.keep_last);
    p.x = a.pooled + ((int64_t)p.layer * a.h_kv + p.g) * a.T + a.tab.cu_seq[p.s];
    p.out = a.idx + ((int64_t)p.layer * a.h_kv + p.g) * a.TB + a.tab.cu_bud[p.s];
    p.hist = a.hist + (((int64_t)p.layer * a.tab.n_seq + p.s) * a.h_kv + p.g) * kHistStride;
    return p;
}

// ------------------------------------------------------------------------------------------------
// general path: one workgroup streams its row three times
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void jq_select_stream_kernel(SelectArgs a) {
    __shared__ uint32_t bins[kHistBins];
    __shared__ uint32_t tmp[kSelectThreads / 64 + 1];
    __shared__ uint32_t res[4];
    const Problem p = problem_of(a, blockIdx.x);
    const float* x = p.x;
    const int L = p.L;

    uint32_t need = p.B;
    pick_bin<kSelectThreads, 2>(p.hist, kHistBins, need, tmp, res);
    const uint32_t b1 = res[0];
    need -= res[1];
    __syncthreads();

    for (int b = threadIdx.x; b < kHistBins; b += kSelectThreads) bins[b] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < L; j += kSelectThreads) {
        const uint32_t k = select_key(x[j], j, L, a.keep_first, a.keep_last);
        if ((k >> 21) == b1) atomicAdd(&bins[(k >> 10) & 2047u], 1u);
    }
    __syncthreads();
    pick_bin<kSelectThreads, 2>(bins, 2048, need, tmp, res);
    const uint32_t prefix22 = (b1 << 11) | res[0];
    need -= res[1];
    __syncthreads();

    for (int b = threadIdx.x; b < 1024; b += kSelectThreads) bins[b] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < L; j += kSelectThreads) {
        const uint32_t k = select_key(x[j], j, L, a.keep_first, a.keep_last);
        if ((k >> 10) == prefix22) atomicAdd(&bins[k & 1023u], 1u);
    }
    __syncthreads();
    pick_bin<kSelectThreads, 1>(bins, 1024, need, tmp, res);
    const uint32_t tau = (prefix22 << 10) | res[0];
    need -= res[1];  // how many elements equal to tau are kept
    __syncthreads();

    // ordered compaction: each thread takes 4 consecutive positions per round
    uint32_t gt_done = 0, eq_done = 0;
    for (int base = 0; base < L; base += kSelectThreads * 4) {
        const int j0 = base + threadIdx.x * 4;
        uint32_t kk[4];
        uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            kk[e] = (j0 + e < L) ? select_key(x[j0 + e], j0 + e, L, a.keep_first, a.keep_last) : 0u;
            n_gt += (j0 + e < L) && kk[e] > tau;
            n_eq += (j0 + e < L) && kk[e] == tau;
        }
        uint32_t total;
        const uint32_t packed = n_gt | (n_eq << 16);  // at most 4096 per field and round
        const uint32_t incl = block_scan_incl<kSelectThreads>(packed, tmp, &total);
        uint32_t gt_before = gt_done + ((incl - packed) & 0xFFFFu);
        uint32_t eq_before = eq_done + ((incl - packed) >> 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (j0 + e >= L) break;
            const bool is_gt = kk[e] > tau, is_eq = kk[e] == tau;
            if (is_gt || (is_eq && eq_before < need)) {
                const uint32_t slot = gt_before + min(eq_before, need);
                if (slot < p.B) p.out[slot] = j0 + e;  // always true for consistent histograms
            }
            gt_before += is_gt;
            eq_before += is_eq;
        }
        gt_done += total & 0xFFFFu;
        eq_done += total >> 16;
        if (gt_done + min(eq_done, need) >= p.B) break;  // uniform: everything kept already
    }
}

// ------------------------------------------------------------------------------------------------
// fast path, step 1: scatter positions above / inside the level-1 threshold bin
// ------------------------------------------------------------------------------------------------
constexpr int kScatterThreads = 256;
constexpr int kScatterPerThread = 8;  // 2048 positions per block (4096: +1.5 us, 1024: +1.5 us on the 128K layer)
constexpr int kScatterBlockPos = kScatterThreads * kScatterPerThread;

__global__ __launch_bounds__(kScatterThreads) void jq_select_scatter_kernel(SelectArgs a) {
    __shared__ uint32_t tmp[kScatterThreads / 64 + 1];
    __shared__ uint32_t res[4];
    __shared__ uint32_t base[2];
    const int g = blockIdx.y, layer = blockIdx.z;
    const int64_t p0 = (int64_t)blockIdx.x * kScatterBlockPos;
    const int64_t p1 = min(a.T, p0 + kScatterBlockPos);
    const int s_first = find_seq(a.tab.cu_seq, a.tab.n_seq, p0);
    const int s_last = find_seq(a.tab.cu_seq, a.tab.n_seq, p1 - 1);
    const float* row = a.pooled + ((int64_t)layer * a.h_kv + g) * a.T;
    // thread t takes positions p0 + t, p0 + t + 256, ...: neighbouring lanes read neighbouring words, and
    // the lists are unordered, so which thread appends which position does not matter
    const int64_t t0 = p0 + threadIdx.x;
    uint32_t key[kScatterPerThread];
#pragma unroll
    for (int e = 0; e < kScatterPerThread; ++e) {
        const int64_t t = t0 + (int64_t)e * kScatterThreads;
        key[e] = (t < p1) ? sortable_key(row[t]) : 0u;
    }

    for (int s = s_first; s <= s_last; ++s) {  // almost always a single sequence
        uint32_t* hist = a.hist + (((int64_t)layer * a.tab.n_seq + s) * a.h_kv + g) * kHistStride;
        const uint32_t B = budget_of(a.layer_budgets, a.tab, layer, s, a.keep_first + a.keep_last);
        const int Ls = a.tab.cu_seq[s + 1] - a.tab.cu_seq[s];
        pick_bin<kScatterThreads, kHistBins / kScatterThreads>(hist, kHistBins, B, tmp, res);
        const uint32_t b1 = res[0];
        const int64_t q0 = max(p0, (int64_t)a.tab.cu_seq[s]), q1 = min(p1, (int64_t)a.tab.cu_seq[s + 1]);
        uint32_t n_s = 0, n_c = 0;
#pragma unroll
        for (int e = 0; e < kScatterPerThread; ++e) {
            const int64_t t = t0 + (int64_t)e * kScatterThreads;
            const bool in = t >= q0 && t < q1;
            const int j = (int)(t - a.tab.cu_seq[s]);
            if (in && (j < a.keep_first || j >= Ls - a.keep_last)) key[e] = 0xFFFFFFFFu;  // always kept
            n_s += in && (key[e] >> 21) > b1;
            n_c += in && (key[e] >> 21) == b1;
        }
        // one pair of global atomics per block: prefix sums inside the block, then a block base
        uint32_t total;
        const uint32_t packed = n_s | (n_c << 16);  // at most kScatterBlockPos per field
        const uint32_t excl = block_scan_incl<kScatterThreads>(packed, tmp, &total) - packed;
        if (threadIdx.x == 0) {
            base[0] = (total & 0xFFFFu) ? atomicAdd(hist + kHistBins, total & 0xFFFFu) : 0u;
            base[1] = (total >> 16) ? atomicAdd(hist + kHistBins + 1, total >> 16) : 0u;
        }
        __syncthreads();
        uint32_t slot_s = base[0] + (excl & 0xFFFFu), slot_c = base[1] + (excl >> 16);
        int32_t* sure = a.sure + ((int64_t)layer * a.h_kv + g) * a.TB + a.tab.cu_bud[s];
        uint2* cand = a.cand + ((int64_t)layer * a.h_kv + g) * a.T + a.tab.cu_seq[s];
#pragma unroll
        for (int e = 0; e < kScatterPerThread; ++e) {
            const int64_t t = t0 + (int64_t)e * kScatterThreads;
            const bool in = t >= q0 && t < q1;
            const uint32_t bin = key[e] >> 21;
            const uint32_t j = (uint32_t)(t - a.tab.cu_seq[s]);
            if (in && bin > b1) { if (slot_s < B) sure[slot_s] = (int32_t)j; ++slot_s; }
            if (in && bin == b1) { if (slot_c < (uint32_t)Ls) cand[slot_c] = make_uint2(key[e], j); ++slot_c; }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// fast path, step 2: resolve the candidates and emit ascending positions
// ------------------------------------------------------------------------------------------------
constexpr int kFinThreads = 512;
constexpr int kFinCache = 16;  // candidates a thread keeps in registers (8192 per block)

__global__ __launch_bounds__(kFinThreads) void jq_select_finalize_kernel(SelectArgs a, int words_cap) {
    extern __shared__ uint32_t lds[];
    uint32_t* bins2 = lds;                        // 2048: level-2 histogram
    uint32_t* bins3 = bins2 + 2048;               // 1024: level-3 histogram
    uint32_t* tmp = bins3 + 1024;                 // scan scratch (padded to 32)
    uint32_t* res = tmp + 32;                     // pick results (padded to 32)
    uint32_t* keep = res + 32;                    // words_cap: bitmap of kept positions
    uint32_t* ties = keep + words_cap;            // words_cap: bitmap of positions with key == tau

    const Problem p = problem_of(a, blockIdx.x);  // blockIdx.y: which slice of the problem's output slots
    const int words = (p.L + 31) >> 5;
    const uint32_t n_sure = min(p.hist[kHistBins], p.B);
    const uint32_t n_cand = min(p.hist[kHistBins + 1], (uint32_t)p.L);
    const int32_t* sure = a.sure + ((int64_t)p.layer * a.h_kv + p.g) * a.TB + a.tab.cu_bud[p.s];
    const uint2* cand = a.cand + ((int64_t)p.layer * a.h_kv + p.g) * a.T + a.tab.cu_seq[p.s];

    // The candidate list is read from global memory once: each thread keeps up to kFinCache entries in
    // registers; anything beyond (huge tie groups) is re-read in every pass.
    uint2 cc[kFinCache];
#pragma unroll
    for (int e = 0; e < kFinCache; ++e) {
        // loaded before the counter is known (the list's storage spans L entries, so this stays in bounds)
        const uint32_t i = threadIdx.x + e * kFinThreads;
        cc[e] = i < (uint32_t)p.L ? cand[i] : make_uint2(0u, 0xFFFFFFFFu);
    }
#pragma unroll
    for (int e = 0; e < kFinCache; ++e)
        if (threadIdx.x + e * kFinThreads >= n_cand) cc[e].y = 0xFFFFFFFFu;  // position 0xFFFFFFFF marks "none"
    const uint32_t spill0 = kFinCache * kFinThreads;
    // the same for the head of the "sure" list (its storage spans B entries)
    constexpr int kSureCache = 4;
    int32_t sc[kSureCache];
#pragma unroll
    for (int e = 0; e < kSureCache; ++e) {
        const uint32_t i = threadIdx.x + e * kFinThreads;
        sc[e] = i < p.B ? sure[i] : 0;
    }

    for (int w = threadIdx.x; w < words; w += kFinThreads) { keep[w] = 0; ties[w] = 0; }
    for (int b = threadIdx.x; b < 3072; b += kFinThreads) bins2[b] = 0;  // both histograms
    __syncthreads();

#pragma unroll
    for (int e = 0; e < kSureCache; ++e) {
        const uint32_t j = (uint32_t)sc[e];
        if (threadIdx.x + e * kFinThreads < n_sure && j < (uint32_t)p.L) atomicOr(&keep[j >> 5], 1u << (j & 31));
    }
    for (uint32_t i = kSureCache * kFinThreads + threadIdx.x; i < n_sure; i += kFinThreads) {
        const uint32_t j = (uint32_t)sure[i];
        if (j < (uint32_t)p.L) atomicOr(&keep[j >> 5], 1u << (j & 31));
    }
    uint32_t need = p.B - n_sure;  // >= 1: the threshold bin always contributes

    // level 2 on the candidates
#pragma unroll
    for (int e = 0; e < kFinCache; ++e)
        if (cc[e].y != 0xFFFFFFFFu) atomicAdd(&bins2[(cc[e].x >> 10) & 2047u], 1u);
    for (uint32_t i = spill0 + threadIdx.x; i < n_cand; i += kFinThreads) atomicAdd(&bins2[(cand[i].x >> 10) & 2047u], 1u);
    __syncthreads();
    pick_bin<kFinThreads, 2048 / kFinThreads>(bins2, 2048, need, tmp, res);
    const uint32_t b2 = res[0];
    need -= res[1];
    // level 3
#pragma unroll
    for (int e = 0; e < kFinCache; ++e)
        if (cc[e].y != 0xFFFFFFFFu && ((cc[e].x >> 10) & 2047u) == b2) atomicAdd(&bins3[cc[e].x & 1023u], 1u);
    for (uint32_t i = spill0 + threadIdx.x; i < n_cand; i += kFinThreads) {
        const uint32_t k = cand[i].x;
        if (((k >> 10) & 2047u) == b2) atomicAdd(&bins3[k & 1023u], 1u);
    }
    __syncthreads();
    pick_bin<kFinThreads, 1024 / kFinThreads>(bins3, 1024, need, tmp, res + 4);
    const uint32_t low21 = (b2 << 10) | res[4];
    need -= res[5];                                   // how many positions with key == tau are kept
    const bool all_ties = (need == res[6]);           // uniform: the whole tie group is kept (the usual case)

    auto classify = [&](uint2 c) {
        const uint32_t k21 = c.x & 0x1FFFFFu;
        if (c.y < (uint32_t)p.L) {
            if (k21 > low21 || (all_ties && k21 == low21)) atomicOr(&keep[c.y >> 5], 1u << (c.y & 31));
            else if (k21 == low21) atomicOr(&ties[c.y >> 5], 1u << (c.y & 31));
        }
    };
#pragma unroll
    for (int e = 0; e < kFinCache; ++e) classify(cc[e]);
    for (uint32_t i = spill0 + threadIdx.x; i < n_cand; i += kFinThreads) classify(cand[i]);
    __syncthreads();

    // thread t owns a contiguous run of words, so thread order is position order
    const int wpt = (words + kFinThreads - 1) / kFinThreads;
    const int w0 = threadIdx.x * wpt, w1 = min(words, w0 + wpt);
    uint32_t total;
    if (!all_ties) {  // the lowest `need` tie positions join the kept set
        uint32_t n_t = 0;
        for (int w = w0; w < w1; ++w) n_t += __popc(ties[w]);
        uint32_t before = block_scan_incl<kFinThreads>(n_t, tmp, &total) - n_t;
        for (int w = w0; w < w1 && before < need; ++w) {
            uint32_t t = ties[w];
            const uint32_t cnt = __popc(t);
            uint32_t take = min(cnt, need - before);
            before += cnt;
            uint32_t add = 0;
            while (take--) { const uint32_t low = t & (0u - t); add |= low; t ^= low; }
            keep[w] |= add;  // only this thread touches word w here
        }
        __syncthreads();
    }
    // Exclusive prefix of the kept count per 32-position word (thread t scans its run of words), then the
    // words are dealt round-robin for emission: kept positions cluster (contiguous heavy-hitter spans), and a
    // thread that owned a whole cluster would emit hundreds of positions alone.
    uint32_t n_k = 0;
    for (int w = w0; w < w1; ++w) n_k += __popc(keep[w]);
    uint32_t run = block_scan_incl<kFinThreads>(n_k, tmp, &total) - n_k;
    uint32_t* wpre = ties;  // the tie bitmap is dead by now
    for (int w = w0; w < w1; ++w) {
        const uint32_t c = __popc(keep[w]);
        wpre[w] = run;
        run += c;
    }
    __syncthreads();
    // Emission is parallel over OUTPUT slots, not over words: kept positions cluster (contiguous heavy-hitter
    // spans), so per-word loops leave most lanes idle.  Slot o lives in the last word w with wpre[w] <= o
    // (binary search in LDS, same trip count for every thread); inside the word, the (o - wpre[w])-th set bit
    // is found by five popcount halvings.  Consecutive threads write consecutive slots.
    const uint32_t per_slice = (p.B + gridDim.y - 1) / gridDim.y;
    const uint32_t o_begin = min(p.B, blockIdx.y * per_slice), o_end = min(p.B, o_begin + per_slice);
    uint32_t* slot_pos = bins2;  // the histograms are dead: positions of the current batch of kFinThreads slots
    for (uint32_t o0 = o_begin; o0 < o_end; o0 += kFinThreads) {  // uniform trip count
        const uint32_t o = o0 + threadIdx.x;
        if (o < o_end) {
            int lo = 0, hi = words;  // invariant: wpre[lo] <= o, and hi == words or wpre[hi] > o
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (wpre[mid] <= o) lo = mid; else hi = mid;
            }
            uint32_t r = o - wpre[lo];
            const uint32_t k = keep[lo];
            uint32_t pos = 0;
#pragma unroll
            for (int sft = 16; sft >= 1; sft >>= 1) {
                const uint32_t c = __popc((k >> pos) & ((1u << sft) - 1u));
                if (r >= c) { r -= c; pos += sft; }
            }
            // (with consistent counts this is a kept position; the clamp keeps the gather inside the sequence whatever
            // the lists hold)
            const uint32_t at = min((uint32_t)(lo << 5) + pos, (uint32_t)p.L - 1u);
            p.out[o] = (int)at;
            slot_pos[threadIdx.x] = at;
        }
        if (a.K_out == nullptr) continue;  // uniform
        // Pruned cache (paper Section 4.3): the kept rows of this batch, 16 lanes x 16 B per 256-byte head row.
        __syncthreads();
        const uint32_t n_rows = min((uint32_t)kFinThreads, o_end - o0);
        const int part = threadIdx.x & 15;
        for (uint32_t rr = threadIdx.x >> 4; rr < n_rows; rr += kFinThreads / 16) {
            const int64_t src = ((kv_row(a.pm, a.tab.cu_seq, a.T, p.layer, p.s, (int)slot_pos[rr]) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
            const int64_t dst = ((kv_row(a.pm_out, a.tab.cu_bud, a.TB, p.layer, p.s, (int)(o0 + rr)) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
            const uint4 kv = *(const uint4*)(a.K + src);
            const uint4 vv = *(const uint4*)(a.V + src);
            *(uint4*)(a.K_out + dst) = kv;
            *(uint4*)(a.V_out + dst) = vv;
        }
        __syncthreads();  // slot_pos is rewritten by the next batch
    }
}

constexpr int kFinalizeFixedWords = 2048 + 1024 + 32 + 32;
constexpr size_t kMaxLds = 160 * 1024;

// Launches of the finalize kernel with more than 64 KiB of dynamic LDS need the function's limit raised.  That
// is done once per device, to the fixed maximum any call can ask for (never to a call's own size: the attribute is
// process-wide, and two host threads with different sequence lengths must not undo each other's setting).
static hipError_t allow_large_lds() {
    static std::atomic<uint64_t> done{0};  // bit d: device d has the limit raised
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute((const void*)jq_select_finalize_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)(kMaxLds - 1024));
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

hipError_t launch_select(const Plan& p, const float* pooled, uint32_t* hist, char* ws, int32_t* idx, hipStream_t st,
                         const void* K, const void* V, void* K_out, void* V_out, bool* gathered) {
    SelectArgs a;
    a.pooled = pooled; a.hist = hist; a.idx = idx;
    a.K = (const char*)K; a.V = (const char*)V; a.K_out = (char*)K_out; a.V_out = (char*)V_out;
    if (gathered) *gathered = false;
    a.sure = (int32_t*)(ws + p.off_sure);
    a.cand = (uint2*)(ws + p.off_cand);
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.T = p.T; a.TB = p.TB;
    a.keep_first = p.keep_first; a.keep_last = p.keep_last;
    a.pm = p.page_map();
    a.pm_out = p.out_map;
    a.layer_budgets = p.layer_budgets;
    a.tab = p.tab;
    const unsigned n_prob = (unsigned)((int64_t)p.n_layers * p.n_seq * p.h_kv);

    int max_len = 0;
    for (int s = 0; s < p.n_seq; ++s) max_len = max(max_len, p.tab.cu_seq[s + 1] - p.tab.cu_seq[s]);
    int words_cap = (max_len + 31) / 32;
    const size_t lds_bytes = ((size_t)kFinalizeFixedWords + 2 * (size_t)words_cap) * sizeof(uint32_t);
    if (lds_bytes > kMaxLds - 1024)  // bitmaps do not fit: stream instead
        return launch_kernel(jq_select_stream_kernel, dim3(n_prob), dim3(kSelectThreads), 0, st, p.marks, kTrFinalize, a);

    dim3 grid((unsigned)((p.T + kScatterBlockPos - 1) / kScatterBlockPos), p.h_kv, p.n_layers);
    hipError_t e = launch_kernel(jq_select_scatter_kernel, grid, dim3(kScatterThreads), 0, st, p.marks, kTrScatter, a);
    if (e != hipSuccess) return e;
    if (lds_bytes > 64 * 1024) {
        e = allow_large_lds();
        if (e != hipSuccess) return e;
    }
    // Slices per problem: enough workgroups to spread the emission (and the gather) over the chip, each with
    // at least 64 output slots.
    int64_t min_budget = INT32_MAX;
    for (int s = 0; s < p.n_seq; ++s) {
        const int64_t b = p.tab.cu_bud[s + 1] - p.tab.cu_bud[s];
        if (b < min_budget) min_budget = b;
    }
    int64_t slices = (256 + n_prob - 1) / n_prob;
    if (slices > (min_budget + 63) / 64) slices = (min_budget + 63) / 64;
    if (slices > 64) slices = 64;
    if (slices < 1) slices = 1;
    if (gathered) *gathered = K_out != nullptr;
    return launch_kernel(jq_select_finalize_kernel, dim3(n_prob, (unsigned)slices), dim3(kFinThreads), lds_bytes, st, p.marks,
                         kTrFinalize, a, words_cap);
}

}  // namespace jq
