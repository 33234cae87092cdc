// Top-B retention per (layer, sequence, KV head): the B best-scored key-value pairs stay, the rest is
// dropped (paper Section 4.3) -- as an exact radix select on the order-preserving 32-bit key of the
// pooled fp32 score.  Ties go to the lower position; output is ascending.
//
//   level 1: bits 31..21, histogram supplied by the pooling kernel                    -> bin b1
//   level 2: bits 20..10 of the elements in b1                                         -> bin b2
//   level 3: bits  9..0  of the elements in (b1, b2)                                   -> threshold key tau
//   result : every key > tau, plus the first (B - #greater) positions with key == tau
//
// Fast path (every sequence of the call fits the LDS bitmaps): ONE kernel after the pooling kernel, which
// has left the best elements of every 1024-position block of the scores as a "segment" of (key, position)
// pairs ordered by level-1 bin, highest first.  A workgroup picks b1 from the histogram, reads each segment
// of its problem until the bins fall below b1 (a few dozen entries per segment; a block with more qualifying
// elements than its segment holds is classified from its pooled scores instead), marks positions above b1 in
// an L-bit LDS bitmap and resolves levels 2 and 3 on the pairs inside b1 (all of them sit in one LDS list),
// marks the chosen positions, trims the tie group to its lowest positions and emits set bits in ascending
// order.  Several workgroups ("slices") work on one problem: each repeats the (cheap, cache-resident)
// resolution and emits its own range of output slots; in the fused eviction call it also gathers the K/V
// rows of those slots, so the pruned cache needs no further kernel.
// General path (very long sequences): one workgroup per problem streams the row three times.
#include <atomic>

#include "jq_common.h"

namespace jq {

struct SelectArgs {
    const float* pooled;  // [n_layers][h_kv][T]
    uint32_t* hist;       // [n_layers][n_seq][h_kv][kHistStride]: level-1 bins
    const uint2* seg;     // [n_layers][h_kv][n_seg][head]  (key, position) by level-1 bin, highest first
    const uint4* seg_hdr; // [n_layers][h_kv][n_seg]  (lowest bin of the block's window, elements inside it, last slot's key, -)
    int32_t head;         // entries kept per segment (a multiple of 64)
    int32_t* idx;         // [n_layers][h_kv][TB]
    // streaming eviction: the cache rows' original positions [n_layers][h_kv][T] and where those of the kept rows
    // go [n_layers][h_kv][TB] (both null otherwise)
    const int32_t* pos_in; int32_t* pos_out;
    int32_t n_layers, h_kv;
    int32_t keep_first, keep_last;  // always-kept positions at either end of every sequence
    int32_t one_L, one_B;           // single-sequence calls: the sequence's length and budget (0 otherwise), next to
                                    // the other scalars, so that a workgroup's first kernel-argument reads do not
                                    // chain through the per-sequence tables further down
    int64_t T, TB;
    // fused gather (all four null when the kept rows are not wanted): K,V [n_layers][T][h_kv][d] bf16,
    // K_out,V_out [n_layers][TB][h_kv][d]
    const char* K; const char* V;
    char* K_out; char* V_out;
    // in-place eviction (dense layouts; K_out, V_out null): kept rows whose source lies inside the front that a later
    // kernel overwrites are copied to `stage` [2][n_layers][TB][h_kv][d] here; that kernel then writes every kept row
    char* stage;
    const uint32_t* dest_bits;  // in-place eviction inside a paged pool: the pages that receive kept rows (else null)
    PageMap pm;      // where the rows of K and V live (dense or paged)
    PageMap pm_out;  // where the kept rows go
    const int32_t* layer_budgets;  // DEVICE [n_layers][n_seq] or null
    int32_t n_seg;                   // segments per layer and head
    int32_t cu_seg[JQ_MAX_SEQ + 1];  // ... per sequence
    SeqTab tab;
};

// bins[0..n_bins): find the bin b with (#elements in bins > b) < need <= (#elements in bins >= b).
// Thread t owns PER consecutive bins, highest bins first.  result[0] = b, result[1] = #elements above,
// result[2] = #elements inside b.
// pick_bin_counts takes the thread's PER counts already loaded (c[e] = count of bin n_bins - 1 - (PER * thread + e)).
template <int THREADS, int PER>
__device__ __forceinline__ void pick_bin_counts(const uint32_t (&c)[PER], int n_bins, uint32_t need, uint32_t* tmp,
                                                uint32_t* result) {
    uint32_t sum = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) sum += c[e];
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
    lds_barrier();
}

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
    lds_barrier();
}

struct Problem {
    int layer, s, g, L;
    int tok0, bud0;  // first token row / first kept row of the sequence (dense layouts)
    uint32_t B;
    const float* x;
    int32_t* out;
    uint32_t* hist;
    const int32_t* pos_in; int32_t* pos_out;  // this problem's slices of the position tables, or null
    __device__ void emit(uint32_t slot, int row) const {
        store_stream(&out[slot], (int32_t)row);
        if (pos_out) store_stream(&pos_out[slot], pos_in[row]);
    }
};

__device__ __forceinline__ Problem problem_of(const SelectArgs& a, int prob) {
    Problem p;
    if (a.one_L) {  // one sequence: nothing to look up
        p.g = prob % a.h_kv;
        p.s = 0;
        p.layer = prob / a.h_kv;
        p.L = a.one_L;
        p.tok0 = 0; p.bud0 = 0;
        p.B = a.layer_budgets ? budget_of(a.layer_budgets, a.tab, p.layer, 0, a.keep_first + a.keep_last) : (uint32_t)a.one_B;
        p.x = a.pooled ? a.pooled + ((int64_t)p.layer * a.h_kv + p.g) * a.T : nullptr;
        p.out = a.idx + ((int64_t)p.layer * a.h_kv + p.g) * a.TB;
        p.hist = a.hist + ((int64_t)p.layer * a.h_kv + p.g) * kHistStride;
        p.pos_in = a.pos_out ? a.pos_in + ((int64_t)p.layer * a.h_kv + p.g) * a.T : nullptr;
        p.pos_out = a.pos_out ? a.pos_out + ((int64_t)p.layer * a.h_kv + p.g) * a.TB : nullptr;
        return p;
    }
    p.g = prob % a.h_kv;
    p.s = (prob / a.h_kv) % a.tab.n_seq;
    p.layer = prob / (a.h_kv * a.tab.n_seq);
    p.L = a.tab.cu_seq[p.s + 1] - a.tab.cu_seq[p.s];
    p.tok0 = a.tab.cu_seq[p.s]; p.bud0 = a.tab.cu_bud[p.s];
    p.B = budget_of(a.layer_budgets, a.tab, p.layer, p.s, a.keep_first + a.keep_last);
    p.x = a.pooled ? a.pooled + ((int64_t)p.layer * a.h_kv + p.g) * a.T + a.tab.cu_seq[p.s] : nullptr;
    p.out = a.idx + ((int64_t)p.layer * a.h_kv + p.g) * a.TB + a.tab.cu_bud[p.s];
    p.hist = a.hist + (((int64_t)p.layer * a.tab.n_seq + p.s) * a.h_kv + p.g) * kHistStride;
    p.pos_in = a.pos_out ? a.pos_in + ((int64_t)p.layer * a.h_kv + p.g) * a.T + a.tab.cu_seq[p.s] : nullptr;
    p.pos_out = a.pos_out ? a.pos_out + ((int64_t)p.layer * a.h_kv + p.g) * a.TB + a.tab.cu_bud[p.s] : nullptr;
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
                if (slot < p.B) p.emit(slot, j0 + e);  // always true for consistent histograms
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
// fast path: resolve the threshold from the sorted segments and emit ascending positions
// ------------------------------------------------------------------------------------------------
constexpr int kFinThreads = 512;
constexpr int kFinWaves = kFinThreads / 64;
constexpr int kSegBatch = 16;  // segments whose first 64 entries a wave requests before it knows the threshold bin

__global__ __launch_bounds__(kFinThreads) void jq_select_finalize_kernel(SelectArgs a, int words_cap, int qual_cap) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    uint32_t* bins2 = lds;                        // 2048: level-2 histogram
    uint32_t* bins3 = bins2 + 2048;               // 1024: level-3 histogram
    uint32_t* tmp = bins3 + 1024;                 // scan scratch (padded to 32)
    uint32_t* res = tmp + 32;                     // pick results (padded to 32)
    uint32_t* cnt = res + 32;                     // [0] elements with bin >= b1 (padded to 32)
    uint32_t* keep = cnt + 32;                    // words_cap: bitmap of kept positions
    uint32_t* ties = keep + words_cap;            // words_cap: bitmap of positions with key == tau
    uint2* qual = (uint2*)(ties + words_cap);     // qual_cap: (key, position) of the elements with bin >= b1
    int32_t* seg_n = (int32_t*)(qual + qual_cap); // segs_cap: usable entries of each segment of the problem (-1: none)

    const Problem p = problem_of(a, blockIdx.x);  // blockIdx.y: which slice of the problem's output slots
    const int words = (p.L + 31) >> 5;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_seg = a.one_L ? a.n_seg : a.cu_seg[p.s + 1] - a.cu_seg[p.s];
    const int64_t seg0 = ((int64_t)p.layer * a.h_kv + p.g) * a.n_seg + (a.one_L ? 0 : a.cu_seg[p.s]);
    const int head = a.head;
    const uint2* segs = a.seg + seg0 * head;
    const uint4* seg_hdr = a.seg_hdr + seg0;

    // Requested first: this thread's four level-1 bins, the header of "its" segment (thread t looks after segment
    // t), and the first entries of the wave's first segments; all of that arrives while the
    // threshold bin is being picked (128 entries of each, two per lane in one 16-byte load: the CU's load path is
    // what bounds this phase, and it counts instructions).  The entry loads are unconditional, from clamped and therefore always valid
    // addresses -- a segment's storage holds `head` entries whatever its element count -- so that all of them are in
    // flight together; what lies outside is masked afterwards.
    uint32_t c1[kHistBins / kFinThreads];
#pragma unroll
    for (int e = 0; e < kHistBins / kFinThreads; ++e) c1[e] = p.hist[kHistBins - 1 - ((kHistBins / kFinThreads) * (int)threadIdx.x + e)];
    const uint4 my_hdr = seg_hdr[min((int)threadIdx.x, n_seg - 1)];
    uint4 ent[kSegBatch];  // entries 2 * lane and 2 * lane + 1 of the wave's i-th segment: (key, position) twice
#pragma unroll
    for (int i = 0; i < kSegBatch; ++i) {
        const uint2* sp = segs + (int64_t)min(wave + i * kFinWaves, n_seg - 1) * head;
        ent[i] = ((const uint4*)sp)[lane];  // one 16-byte load per lane covers the segment's first 128 entries
    }
    for (int w = 4 * threadIdx.x; w < 2 * words_cap; w += 4 * kFinThreads) *(uint4*)&keep[w] = make_uint4(0u, 0u, 0u, 0u);  // keep, ties
    for (int b = 4 * threadIdx.x; b < 3072 + 96; b += 4 * kFinThreads) *(uint4*)&bins2[b] = make_uint4(0u, 0u, 0u, 0u);  // histograms, tmp, res, cnt
    lds_barrier();
    pick_bin_counts<kFinThreads, kHistBins / kFinThreads>(c1, kHistBins, p.B, tmp, res);
    const uint32_t b1 = res[0];
    const uint32_t n_above = res[1];  // positions above bin b1 (all of them are kept); < B

    // header = (lowest bin of the block's window, elements inside the window, key of the segment's last slot);
    // usable entries of a segment, or -1 when the segment cannot answer -- more qualifying elements than it holds,
    // or a window that ends above b1 -- and the block is classified from its pooled scores instead
    auto usable = [&](uint4 hdr) {
        const bool answers = b1 >= hdr.x && !((int)hdr.y > head && (hdr.z >> 21) >= b1);
        return answers ? min(head, (int)hdr.y) : -1;
    };
    for (int t = threadIdx.x; t < n_seg; t += kFinThreads) seg_n[t] = usable(t == (int)threadIdx.x ? my_hdr : seg_hdr[t]);
    lds_barrier();

    // Every entry with bin >= b1 goes into one flat LDS list `qual` (as far as it reaches; cnt[0] counts them all),
    // which the passes below work through evenly, a few entries per thread.  The entries of a wave's first segments
    // are counted with ballots first, so that the whole batch needs ONE reservation: atomics of many lanes on one
    // LDS word are served one at a time.
    auto put = [&](uint32_t key, uint32_t pos) __attribute__((always_inline)) {  // rare paths: one reservation per entry
        const uint32_t to = atomicAdd(&cnt[0], 1u);
        if (to < (uint32_t)qual_cap) qual[to] = make_uint2(key, pos);
    };
    auto scan_block = [&](int sg, auto f) __attribute__((always_inline)) {
        const int j0 = sg * kSegLen, j1 = min(p.L, j0 + kSegLen);
        for (int j = j0 + lane; j < j1; j += 64) {
            const uint32_t key = select_key(p.x[j], j, p.L, a.keep_first, a.keep_last);
            if ((key >> 21) >= b1) f(key, (uint32_t)j);
        }
    };
    const int my_n = seg_n[min(wave + (lane & (kSegBatch - 1)) * kFinWaves, n_seg - 1)];  // lane i < 16: the wave's i-th segment
    uint64_t ge_even[kSegBatch], ge_odd[kSegBatch];  // wave-uniform: lanes whose even / odd entry of the i-th segment qualifies
    uint32_t n_mine = 0, again = 0;                  // again, bit i: the 128th entry of the i-th segment still qualified
#pragma unroll
    for (int i = 0; i < kSegBatch; ++i) {
        const int n = wave + i * kFinWaves < n_seg ? __builtin_amdgcn_readlane(my_n, i) : 0;  // -1: not from its entries
        ge_even[i] = __ballot(2 * lane < n && (ent[i].x >> 21) >= b1);
        ge_odd[i] = __ballot(2 * lane + 1 < n && (ent[i].z >> 21) >= b1);
        n_mine += (uint32_t)(__popcll(ge_even[i]) + __popcll(ge_odd[i]));
        again |= (uint32_t)(ge_odd[i] >> 63) << i;
    }
    if (n_mine) {  // wave-uniform
        uint32_t to = 0;
        if (lane == 0) to = atomicAdd(&cnt[0], n_mine);
        to = __builtin_amdgcn_readfirstlane(to);
#pragma unroll
        for (int i = 0; i < kSegBatch; ++i) {
            const uint64_t me = ge_even[i], mo = ge_odd[i];
            const uint32_t se = to + __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0u));
            if (((me >> lane) & 1) && se < (uint32_t)qual_cap) qual[se] = make_uint2(ent[i].x, ent[i].y);
            to += (uint32_t)__popcll(me);
            const uint32_t so = to + __builtin_amdgcn_mbcnt_hi((uint32_t)(mo >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mo, 0u));
            if (((mo >> lane) & 1) && so < (uint32_t)qual_cap) qual[so] = make_uint2(ent[i].z, ent[i].w);
            to += (uint32_t)__popcll(mo);
        }
    }
    // Second visits (a segment whose 128th entry still qualified, a block that is classified from its scores), and
    // the segments beyond the first batch: rare, so the common case only tests one mask.
    auto visit = [&](int sg, int n, int off) __attribute__((always_inline)) {
        if (n < 0) {
            scan_block(sg, put);
            return;
        }
        // chunks of 64 entries while the previous chunk's last entry still qualified
        bool last_in = true;
        for (; off < n && last_in; off += 64) {
            const uint2 e = segs[(int64_t)sg * head + min(off + lane, head - 1)];
            const bool ge = off + lane < n && (e.x >> 21) >= b1;
            if (ge) put(e.x, e.y);
            last_in = (__ballot(ge) >> 63) != 0;
        }
    };
    again |= (uint32_t)__ballot(lane < kSegBatch && wave + lane * kFinWaves < n_seg && my_n < 0);
    while (again) {  // wave-uniform
        const int i = __builtin_ctz(again);
        again &= again - 1;
        const int sg = wave + i * kFinWaves;
        visit(sg, seg_n[sg], 128);
    }
    for (int sg = wave + kSegBatch * kFinWaves; sg < n_seg; sg += kFinWaves) visit(sg, seg_n[sg], 0);
    lds_barrier();
    const uint32_t n_qual = cnt[0];
    const bool listed = n_qual <= (uint32_t)qual_cap;  // uniform; otherwise every pass re-reads the scores
    uint32_t need = p.B - min(n_above, p.B - 1);       // >= 1: the threshold bin always contributes

    // f(key, position) for every element with bin >= b1
    auto for_each_qual = [&](auto f) __attribute__((always_inline)) {
        if (listed) {
            for (uint32_t i = threadIdx.x; i < n_qual; i += kFinThreads) f(qual[i].x, qual[i].y);
        } else {
            for (int sg = wave; sg < n_seg; sg += kFinWaves) scan_block(sg, f);
        }
    };
    // positions above b1 are kept; level 2 on the pairs inside b1
    for_each_qual([&](uint32_t key, uint32_t pos) {
        if (pos >= (uint32_t)p.L) return;
        if ((key >> 21) > b1) atomicOr(&keep[pos >> 5], 1u << (pos & 31));
        else atomicAdd(&bins2[(key >> 10) & 2047u], 1u);
    });
    lds_barrier();
    pick_bin<kFinThreads, 2048 / kFinThreads>(bins2, 2048, need, tmp, res);
    const uint32_t b2 = res[0];
    need -= res[1];
    // level 3
    for_each_qual([&](uint32_t key, uint32_t pos) {
        if (pos < (uint32_t)p.L && (key >> 10) == ((b1 << 11) | b2)) atomicAdd(&bins3[key & 1023u], 1u);
    });
    lds_barrier();
    pick_bin<kFinThreads, 1024 / kFinThreads>(bins3, 1024, need, tmp, res + 4);
    const uint32_t tau = (((b1 << 11) | b2) << 10) | res[4];
    need -= res[5];                                   // how many positions with key == tau are kept
    const bool all_ties = (need == res[6]);           // uniform: the whole tie group is kept (the usual case)
    for_each_qual([&](uint32_t key, uint32_t pos) {
        if (pos >= (uint32_t)p.L || (key >> 21) != b1) return;
        if (key > tau || (all_ties && key == tau)) atomicOr(&keep[pos >> 5], 1u << (pos & 31));
        else if (key == tau) atomicOr(&ties[pos >> 5], 1u << (pos & 31));
    });
    lds_barrier();

    // Thread t owns a contiguous run of `wpt` words (a multiple of four, read as 16-byte vectors; the bitmaps are
    // padded with zero words up to kFinThreads * wpt), so thread order is position order.
    const int wpt = words_cap / kFinThreads;
    const int w0 = threadIdx.x * wpt;
    uint32_t total;
    if (!all_ties) {  // the lowest `need` tie positions join the kept set
        uint32_t n_t = 0;
        for (int w = w0; w < w0 + wpt; ++w) n_t += __popc(ties[w]);
        uint32_t before = block_scan_incl<kFinThreads>(n_t, tmp, &total) - n_t;
        for (int w = w0; w < w0 + wpt && before < need; ++w) {
            uint32_t t = ties[w];
            const uint32_t cnt_w = __popc(t);
            uint32_t take = min(cnt_w, need - before);
            before += cnt_w;
            uint32_t add = 0;
            while (take--) { const uint32_t low = t & (0u - t); add |= low; t ^= low; }
            keep[w] |= add;  // only this thread touches word w here
        }
        lds_barrier();
    }
    // Exclusive prefix of the kept count per 32-position word.
    uint32_t n_k = 0;
    for (int w = w0; w < w0 + wpt; w += 4) {
        const uint4 k4 = *(const uint4*)&keep[w];
        n_k += __popc(k4.x) + __popc(k4.y) + __popc(k4.z) + __popc(k4.w);
    }
    uint32_t run = block_scan_incl<kFinThreads>(n_k, tmp, &total) - n_k;
    uint32_t* wpre = ties;  // the tie bitmap is dead by now
    for (int w = w0; w < w0 + wpt; w += 4) {
        const uint4 k4 = *(const uint4*)&keep[w];
        uint4 pre;
        pre.x = run; run += __popc(k4.x);
        pre.y = run; run += __popc(k4.y);
        pre.z = run; run += __popc(k4.z);
        pre.w = run; run += __popc(k4.w);
        *(uint4*)&wpre[w] = pre;
    }
    lds_barrier();
    const uint32_t per_slice = (p.B + gridDim.y - 1) / gridDim.y;
    const uint32_t o_begin = min(p.B, blockIdx.y * per_slice), o_end = min(p.B, o_begin + per_slice);
    uint32_t* slot_pos = bins2;  // the histograms are dead: kept positions of (a batch of) the slice's output slots
    // Pruned cache (paper Section 4.3): the kept rows of output slots o0 .. o0 + n_rows - 1, whose positions are in
    // slot_pos; 16 lanes x 16 B per 256-byte head row.
    auto gather_rows = [&](uint32_t o0, uint32_t n_rows) __attribute__((always_inline)) {
        const int part = threadIdx.x & 15;
        if (a.stage) {  // uniform
            const int64_t v_stage = (int64_t)a.n_layers * a.TB * a.h_kv * (kHeadDim * 2);
            for (uint32_t rr = threadIdx.x >> 4; rr < n_rows; rr += kFinThreads / 16) {
                const int64_t src_row = (int64_t)p.tok0 + slot_pos[rr];  // within the layer (dense layout)
                if (!row_is_overwritten(a.pm, a.dest_bits, src_row, a.TB, p.s, (int)slot_pos[rr])) continue;  // read in place later
                const int64_t src = ((kv_row_from(a.pm, p.tok0, a.T, p.layer, p.s, (int)slot_pos[rr]) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
                const int64_t stg = ((((int64_t)p.layer * a.TB + p.bud0 + o0 + rr) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
                *(uint4*)(a.stage + stg) = *(const uint4*)(a.K + src);
                *(uint4*)(a.stage + v_stage + stg) = *(const uint4*)(a.V + src);
            }
            return;
        }
        for (uint32_t rr = threadIdx.x >> 4; rr < n_rows; rr += kFinThreads / 16) {
            const int64_t src = ((kv_row_from(a.pm, p.tok0, a.T, p.layer, p.s, (int)slot_pos[rr]) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
            const int64_t dst = ((kv_row_from(a.pm_out, p.bud0, a.TB, p.layer, p.s, (int)(o0 + rr)) * a.h_kv + p.g) * kHeadDim) * 2 + part * 16;
            const uint4 kv = *(const uint4*)(a.K + src);
            const uint4 vv = *(const uint4*)(a.V + src);
            store_stream16(a.K_out + dst, kv);
            store_stream16(a.V_out + dst, vv);
        }
    };
    const bool want_rows = a.K_out != nullptr || a.stage != nullptr;  // uniform
    if (listed && o_end - o_begin <= 3072u) {
        // Every kept element sits in the flat list, and its output slot is its rank among the kept positions:
        // the words before its own (prefix array) plus the set bits below it in its word.
        for (uint32_t i = threadIdx.x; i < n_qual; i += kFinThreads) {
            const uint32_t pos = qual[i].y;
            if (pos >= (uint32_t)p.L) continue;
            const uint32_t word = keep[pos >> 5], bit = pos & 31;
            if (!((word >> bit) & 1u)) continue;
            const uint32_t o = wpre[pos >> 5] + __popc(word & ((1u << bit) - 1u));
            if (o >= o_begin && o < o_end) {
                p.emit(o, (int)pos);
                slot_pos[o - o_begin] = pos;
            }
        }
        if (!want_rows) return;  // uniform
        lds_barrier();
        gather_rows(o_begin, o_end - o_begin);
        return;
    }
    // Otherwise emission is parallel over OUTPUT slots: slot o lives in the last word w with wpre[w] <= o (binary
    // search in LDS, same trip count for every thread); inside the word, the (o - wpre[w])-th set bit is found by
    // five popcount halvings.  Consecutive threads write consecutive slots.
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
            p.emit(o, (int)at);
            slot_pos[threadIdx.x] = at;
        }
        if (!want_rows) continue;  // uniform
        lds_barrier();
        gather_rows(o0, min((uint32_t)kFinThreads, o_end - o0));
        lds_barrier();  // slot_pos is rewritten by the next batch
    }
}

constexpr int kFinalizeFixedWords = 2048 + 1024 + 32 + 32 + 32;
constexpr size_t kMaxLds = 160 * 1024;
constexpr int kQualCap = 8192;     // elements at or above the threshold bin that the LDS list holds when there is room
constexpr int kQualCapMin = 1024;

// LDS of the finalize kernel for the plan's longest sequence: the two bitmaps, one word per segment, then as much
// list as fits.
static size_t finalize_lds(const Plan& p, int* words_cap, int* qual_cap) {
    int max_len = 0;
    for (int s = 0; s < p.n_seq; ++s) max_len = max(max_len, p.tab.cu_seq[s + 1] - p.tab.cu_seq[s]);
    *words_cap = ((max_len + 31) / 32 + 4 * kFinThreads - 1) / (4 * kFinThreads) * (4 * kFinThreads);  // whole 16-byte vectors per thread
    const size_t segs_cap = ((size_t)max_len + kSegLen - 1) / kSegLen;
    const size_t fixed = ((size_t)kFinalizeFixedWords + 2 * (size_t)*words_cap + segs_cap) * sizeof(uint32_t);
    const size_t room = kMaxLds - 1024 > fixed ? (kMaxLds - 1024 - fixed) / sizeof(uint2) : 0;
    *qual_cap = (int)(room < (size_t)kQualCap ? room : (size_t)kQualCap);
    return fixed + (size_t)*qual_cap * sizeof(uint2);
}

bool select_fast_path(const Plan& p) {
    int words_cap, qual_cap;
    finalize_lds(p, &words_cap, &qual_cap);
    return qual_cap >= kQualCapMin;  // otherwise the bitmaps (nearly) fill LDS: stream instead
}

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
                         const void* K, const void* V, void* K_out, void* V_out, bool* gathered, void* stage,
                         const int32_t* pos_in, int32_t* pos_out, const uint32_t* dest_bits) {
    SelectArgs a;
    a.dest_bits = dest_bits;
    a.pooled = pooled; a.hist = hist; a.idx = idx;
    a.pos_in = pos_in; a.pos_out = pos_out;
    a.K = (const char*)K; a.V = (const char*)V; a.K_out = (char*)K_out; a.V_out = (char*)V_out;
    a.stage = (char*)stage;
    if (gathered) *gathered = false;
    a.seg = (const uint2*)(ws + p.off_seg);
    a.seg_hdr = (const uint4*)(ws + p.off_seghdr);
    a.head = p.seg_head;
    a.n_layers = p.n_layers; a.h_kv = p.h_kv; a.T = p.T; a.TB = p.TB;
    a.keep_first = p.keep_first; a.keep_last = p.keep_last;
    a.one_L = p.n_seq == 1 ? p.tab.cu_seq[1] : 0;
    a.one_B = p.n_seq == 1 ? p.tab.cu_bud[1] : 0;
    a.pm = p.page_map();
    a.pm_out = p.out_map;
    a.layer_budgets = p.layer_budgets;
    a.n_seg = p.n_seg;
    for (int s = 0; s <= p.n_seq; ++s) a.cu_seg[s] = p.cu_seg[s];
    a.tab = p.tab;
    const unsigned n_prob = (unsigned)((int64_t)p.n_layers * p.n_seq * p.h_kv);

    if (!select_fast_path(p))  // bitmaps do not fit: stream instead
        return launch_kernel(jq_select_stream_kernel, dim3(n_prob), dim3(kSelectThreads), 0, st, p.marks, kTrFinalize, a);

    int words_cap, qual_cap;
    const size_t lds_bytes = finalize_lds(p, &words_cap, &qual_cap);
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_large_lds();
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
    if (gathered) *gathered = K_out != nullptr || stage != nullptr;
    return launch_kernel(jq_select_finalize_kernel, dim3(n_prob, (unsigned)slices), dim3(kFinThreads), lds_bytes, st, p.marks,
                         kTrFinalize, a, words_cap, qual_cap);
}

}  // namespace jq
